"""GPU parity: libstar (through its C ABI) against the CPU oracle, element by
element, on seeded inputs small enough for the oracle yet spanning many
workgroups, several chunks per thread and a ragged tail."""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
import workloads
from oracle import star_oracle as so
from gpu_util import TOL, TOL_BF16_OBSERVED, gpu_update, opts, rand_rows, rand_stream, tile_order, to_dev_rows  # noqa: F401 (tile_order: autouse fixture)

pytestmark = pytest.mark.gpu

KERNELS = {"auto": star.KERNEL_AUTO, "seq": star.KERNEL_SEQ, "affine": star.KERNEL_AFFINE,
           "mfma": star.KERNEL_AFFINE_MFMA}


def check(p, v, n, ep, ev, en, dtype, what=""):
    tol = min(TOL[dtype], TOL_BF16_OBSERVED)
    e_p, e_v = so.max_rel_err(p, ep), so.max_rel_err(v, ev)
    print(f"[{what}] err p={e_p:.3g} v={e_v:.3g}", end="")
    assert e_p <= tol and e_v <= tol, (what, e_p, e_v)
    if en is not None:
        e_n = float(np.max(np.abs(n - en) / np.maximum(np.abs(en), 1e-30))) if len(en) else 0.0
        print(f" norms={e_n:.3g}", end="")
        assert e_n <= tol, (what, e_n)
    print(flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kname", ["seq", "affine", "auto", "mfma"])
@pytest.mark.parametrize("W,P,U,norms", [
    (1, 1, 1, True), (2, 3, 2, False), (4, 5, 10, True), (3, 1023, 7, True), (5, 1025, 12, False),
    (8, 4099, 24, True), (16, 70001, 16, True), (17, 33333, 9, True), (32, 50000, 12, False),
    (32, 20003, 6, True), (12, 600011, 20, True),
    # short streams (the step-by-step kernel is queue-ordered up to 2 updates) and shards of more tiles than
    # the first, fixed round of claims covers (256 or 512 workgroups x 2 tiles on average)
    (8, 300007, 2, True), (16, 1300003, 3, True), (16, 1300003, 16, True), (6, 1100000, 1, False),
    # streams that the step-by-step kernel splits over two launches although their tables are small
    (8, 4099, 32, True), (8, 4099, 30, True), (1, 4099, 32, True),
])
def test_random_shapes(dtype, kname, W, P, U, norms):
    rng = np.random.default_rng(1000 * W + U + (7 if dtype == "bf16" else 0))
    rows = rand_rows(rng, W, P, dtype)
    offs, mem, st = rand_stream(rng, W, U, stale=4)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    print(f"case W={W} P={P} U={U} norms={norms} {dtype} {kname}", flush=True)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, staleness=st, want_norms=norms, **hp)
    p, v, n = gpu_update(p0, v0, rows, offs, mem, staleness=st, want_norms=norms, kernel=KERNELS[kname], **hp)
    check(p, v, n, ep, ev, en, dtype, f"{kname} W={W} P={P} U={U}")


@pytest.mark.parametrize("seed", range(6))
def test_random_calls_whatever_the_library_chooses(seed):
    """Random calls -- row count, stream length, group sizes, dtype, shard length up to 2.5 Mi elements, weighting,
    norms, the direct-norms flag, either entry point -- with the library left to choose its kernels: whichever
    of its rules fires (literal kernel for very short streams, vector-register or matrix-core Gram, even split,
    direct norm pass, collapsed update with the norm walk), the result is the oracle's."""
    rng = np.random.default_rng(5000 + seed)
    for case in range(12):
        W = int(rng.choice([1, 2, 3, 5, 6, 7, 8, 9, 12, 16, 17, 24, 32]))
        U = int(rng.choice([1, 2, 3, 4, 6, 10, 24]))
        P = int(rng.choice([1, 77, 4099, 70001, 300007, 1300003, 2500001]))
        if P > 1000000 and W * U > 200:
            P = 300007                    # keeps the oracle's share of the test at seconds
        dtype = str(rng.choice(["f32", "bf16"]))
        norms = bool(rng.random() < 0.7)
        wmode = str(rng.choice(["mean", "stale", "explicit"]))
        rows = rand_rows(rng, W, P, dtype)
        offs, mem, st = rand_stream(rng, W, U, max_y=int(rng.integers(1, W + 1)), stale=3)
        cf = None
        if wmode == "explicit":
            cf = rng.uniform(0.05, 1.0, len(mem)).astype(np.float32)
        hp = dict(lr=0.05, momentum_coef=float(rng.choice([0.0, 0.9])), weight_decay=float(rng.choice([0.0, 1e-3])),
                  wmode=wmode, scale_lr_by_group=bool(rng.random() < 0.3))
        stale = st if wmode == "stale" else None
        p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
        v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)
        direct = bool(norms and rng.random() < 0.25)
        noalloc = bool(rng.random() < 0.3)
        us = star.UpdateStream(offs, mem, stale, cf)
        c = star.star_plan_choice(P, W, dtype, us, want_norms=norms, direct_norms=direct, **hp)
        what = (f"seed {seed} case {case}: W={W} U={U} P={P} {dtype} norms={norms} {wmode} direct={direct} noalloc={noalloc} "
                f"-> kernel {c['kernel']} collapsed {c['collapsed_update']} launches {c['launches']}")
        print(what, flush=True)
        ep, ev, en = so.group_update(p0, v0, rows, offs, mem, staleness=stale, coeff=cf, want_norms=norms, **hp)
        p, v = torch.from_numpy(p0).cuda(), torch.from_numpy(v0).cuda()
        n = torch.full((U,), -1.0, device="cuda") if norms else None
        if noalloc:
            star.star_group_update_noalloc(p, v, to_dev_rows(rows), us, norms_out=n, **hp)
        else:
            star.star_group_update(p, v, to_dev_rows(rows), us, norms_out=n, direct_norms=direct, **opts(), **hp)
        torch.cuda.synchronize()
        check(p.cpu().numpy(), v.cpu().numpy(), None if n is None else n.cpu().numpy(), ep, ev, en, dtype, what)


@pytest.mark.parametrize("name", workloads.ORDER)
@pytest.mark.parametrize("kname", ["seq", "auto"])
def test_workload_structure_scaled_down(name, kname):
    """Each of the five workloads with its own W, dtype, group mix, weights and
    hyper-parameters, at a shard length the oracle finishes in seconds."""
    wl = workloads.WORKLOADS[name].scaled(262144 + 4 * 257 + 3)
    p0 = workloads.make_params(wl, 0).numpy()
    p, v = p0.copy(), np.zeros_like(p0)
    ep, ev = p0.copy(), np.zeros_like(p0)
    print(f"workload {name} {kname}", flush=True)
    rows = None
    for call in range(wl.calls):
        if rows is None or wl.fresh_grads_per_call:
            rows = workloads.rows_to_numpy(workloads.make_grad_rows(wl, 0, call))
        s = workloads.make_update_stream(wl, 0, call)
        hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
        ep, ev, en = so.group_update(ep, ev, rows, s["offsets"], s["members"], staleness=s["staleness"],
                                     want_norms=wl.norms, **hp)
        p, v, n = gpu_update(p, v, rows, s["offsets"], s["members"], staleness=s["staleness"], want_norms=wl.norms,
                             kernel=KERNELS[kname], **hp)
        check(p, v, n, ep, ev, en, wl.grad_dtype, f"{name} call {call} {kname}")


def test_member_order_is_bitwise_irrelevant():
    rng = np.random.default_rng(5)
    W, P, U = 9, 10007, 11
    rows = rand_rows(rng, W, P, "f32")
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = rng.standard_normal(P).astype(np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale", want_norms=True)
    mem2, st2 = mem.copy(), st.copy()
    for u in range(U):
        perm = rng.permutation(offs[u + 1] - offs[u]) + offs[u]
        mem2[offs[u]:offs[u + 1]], st2[offs[u]:offs[u + 1]] = mem[perm], st[perm]
    for k in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        a = gpu_update(p0, v0, rows, offs, mem, staleness=st, kernel=k, **hp)
        b = gpu_update(p0, v0, rows, offs, mem2, staleness=st2, kernel=k, **hp)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_run_to_run_bitwise_reproducible():
    """Params and momentum are the same bits every run.  So are the norms, also when the tiles come from
    the queue and every run hands them to the workgroups differently: the sums across tiles are carried
    in double, where that order shows only at 1e-16, far below the fp32 result."""
    rng = np.random.default_rng(6)
    W, P = 16, 900001
    rows = rand_rows(rng, W, P, "bf16")
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale", want_norms=True)
    for k, U in ((star.KERNEL_SEQ, 3), (star.KERNEL_SEQ, 20), (star.KERNEL_AFFINE, 20), (star.KERNEL_AFFINE_MFMA, 20)):
        offs, mem, st = rand_stream(rng, W, U, stale=3)
        a = gpu_update(p0, v0, rows, offs, mem, staleness=st, kernel=k, **hp)
        for _ in range(3):
            b = gpu_update(p0, v0, rows, offs, mem, staleness=st, kernel=k, **hp)
            for x, y in zip(a, b):
                assert np.array_equal(x, y)


def test_batch_split_carries_state():
    """One call with U updates against two calls with U1 + U2.  Both evaluations agree to rounding: the
    collapsed one rounds once per call, the step-by-step one carries the low part of the parameters
    from update to update within a call and drops it at the call boundary (at most an ulp).  The
    step-by-step norms do not depend on the state and must agree bit for bit."""
    rng = np.random.default_rng(7)
    W, P, U, k = 6, 50001, 14, 5
    rows = rand_rows(rng, W, P, "f32")
    offs, mem, _ = rand_stream(rng, W, U)
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = rng.standard_normal(P).astype(np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, want_norms=True)
    for kern, exact in ((star.KERNEL_SEQ, True), (star.KERNEL_AFFINE, False)):
        p, v, n = gpu_update(p0, v0, rows, offs, mem, kernel=kern, **hp)
        pa, va, na = gpu_update(p0, v0, rows, offs[:k + 1], mem[:offs[k]], kernel=kern, **hp)
        pb, vb, nb = gpu_update(pa, va, rows, offs[k:] - offs[k], mem[offs[k]:], kernel=kern, **hp)
        if exact:
            assert so.max_rel_err(pb, p) < 2e-7 and so.max_rel_err(vb, v) < 2e-7
            assert np.array_equal(n, np.concatenate([na, nb]))
        else:
            assert so.max_rel_err(pb, p) < 1e-6 and so.max_rel_err(vb, v) < 1e-6
            np.testing.assert_allclose(np.concatenate([na, nb]), n, rtol=1e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unaligned_buffers_give_identical_results(dtype):
    rng = np.random.default_rng(8)
    W, P, U = 5, 40009, 8
    rows = rand_rows(rng, W, P + 3, dtype)
    offs, mem, _ = rand_stream(rng, W, U)
    p0 = rng.standard_normal(P + 3).astype(np.float32)
    v0 = rng.standard_normal(P + 3).astype(np.float32)
    us = star.UpdateStream(offs, mem)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3)
    for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        for shift in (0, 1):          # shift 1: every base pointer is off the 16-byte grid
            drows = [r[shift:shift + P].clone() if shift == 0 else r[shift:shift + P] for r in to_dev_rows(rows)]
            rows_same = [r[0:P] for r in rows] if shift == 0 else [r[1:1 + P] for r in rows]
            p = torch.from_numpy(p0).cuda()[shift:shift + P]
            v = torch.from_numpy(v0).cuda()[shift:shift + P]
            if shift == 0:
                p, v = p.clone(), v.clone()
            n = torch.zeros(U, device="cuda")
            star.star_group_update(p, v, drows, us, norms_out=n, **opts(kern), **hp)
            torch.cuda.synchronize()
            ep, ev, en = so.group_update(p0[shift:shift + P], v0[shift:shift + P], rows_same, offs, mem,
                                         want_norms=True, **hp)
            check(p.cpu().numpy(), v.cpu().numpy(), n.cpu().numpy(), ep, ev, en, dtype, f"shift {shift}")


def test_norms_entry_point_matches_update_norms():
    rng = np.random.default_rng(9)
    for W, P, U, dtype in ((7, 123457, 10, "f32"), (16, 90001, 30, "bf16"), (24, 30011, 8, "f32")):
        rows = rand_rows(rng, W, P, dtype)
        offs, mem, st = rand_stream(rng, W, U, stale=5)
        en = so.group_norms(rows, offs, mem, wmode="stale", staleness=st)
        drows = to_dev_rows(rows)
        us = star.UpdateStream(offs, mem, st)
        for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE, star.KERNEL_AUTO, star.KERNEL_AFFINE_MFMA):
            n = torch.full((U,), -1.0, device="cuda")
            star.star_group_norms(drows, us, n, wmode="stale", **opts(kern))
            torch.cuda.synchronize()
            err = np.max(np.abs(n.cpu().numpy() - en) / en)
            print(f"norms-only W={W} kern={kern} err={err:.3g}", flush=True)
            assert err <= TOL[dtype]


def test_long_stream_is_chunked():
    """More updates than one launch of the step-by-step kernel holds."""
    rng = np.random.default_rng(10)
    W, P, U = 4, 9001, 300
    rows = rand_rows(rng, W, P, "f32", std=1e-3)
    offs, mem, _ = rand_stream(rng, W, U)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=0.01, momentum_coef=0.9, weight_decay=1e-4, want_norms=True)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, **hp)
    for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        p, v, n = gpu_update(p0, v0, rows, offs, mem, kernel=kern, **hp)
        e_p, e_v = so.max_rel_err(p, ep), so.max_rel_err(v, ev)
        print(f"U=300 kern={kern}: err p={e_p:.3g} v={e_v:.3g}", flush=True)
        assert e_p <= 1e-6 and e_v <= 1e-6     # the literal form carries the low part of p from update to update
        np.testing.assert_allclose(n, en, rtol=1e-6)


def test_special_modes_explicit_coefficients_scaled_lr_per_update_lr():
    rng = np.random.default_rng(11)
    W, P, U = 8, 20001, 9
    rows = rand_rows(rng, W, P, "f32")
    offs, mem, _ = rand_stream(rng, W, U)
    cf = rng.uniform(-1, 1, len(mem)).astype(np.float32)
    lrs = rng.uniform(0.01, 0.1, U).astype(np.float32)
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = rng.standard_normal(P).astype(np.float32)
    hp = dict(lr=0.3, momentum_coef=0.8, weight_decay=1e-2, wmode="explicit", scale_lr_by_group=True, want_norms=True)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, coeff=cf, lr_per_update=lrs, **hp)
    for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        p, v, n = gpu_update(p0, v0, rows, offs, mem, coeff=cf, lr_per_update=lrs, kernel=kern, **hp)
        check(p, v, n, ep, ev, en, "f32", f"explicit kern={kern}")


def test_unreferenced_rows_may_be_null():
    rng = np.random.default_rng(12)
    W, P = 6, 5003
    rows = rand_rows(rng, W, P, "f32")
    offs, mem = np.array([0, 2, 3], np.int32), np.array([4, 1, 4], np.int32)
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.0, want_norms=True)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, **hp)
    sparse = [r if w in (1, 4) else None for w, r in enumerate(rows)]
    for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        p, v, n = gpu_update(p0, v0, sparse, offs, mem, kernel=kern, **hp)
        check(p, v, n, ep, ev, en, "f32", f"null rows kern={kern}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rows_marshalled_once_give_the_same_bits(dtype):
    """GradRows (the rows' pointers marshalled once, for callers that reuse their buffers) against the plain
    list of tensors: the same call, so the same bits, for every entry point that takes rows; unused rows may
    be None in it too; a shard length that does not match is refused."""
    rng = np.random.default_rng(21)
    W, P, U = 6, 70001, 5
    rows_np = rand_rows(rng, W, P, dtype)
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    us = star.UpdateStream(offs, mem, st)
    drows = to_dev_rows(rows_np)
    used = set(int(x) for x in mem)
    sparse = [r if w in used else None for w, r in enumerate(drows)]
    held = star.GradRows(sparse)
    assert len(held) == W and held.P == P
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    res = []
    for r in (drows, held):
        p = torch.from_numpy((np.arange(P) % 7 * 0.01).astype(np.float32)).cuda()
        v = torch.zeros(P, device="cuda")
        n, n2, nr = torch.zeros(U, device="cuda"), torch.zeros(U, device="cuda"), torch.zeros(U, device="cuda")
        out = [torch.zeros(P, device="cuda", dtype=drows[0].dtype) for _ in range(U)]
        star.star_group_update(p, v, r, us, norms_out=n, **opts(), **hp)
        star.star_group_norms(r, us, n2, wmode="stale", **opts())
        star.star_group_reduce(out, r, us, wmode="stale", norms_out=nr, **opts())
        torch.cuda.synchronize()
        res.append([p, v, n, n2, nr] + out)
    for a, b in zip(*res):
        assert torch.equal(a, b)
    with pytest.raises(ValueError):
        star.star_group_update(torch.zeros(P + 1, device="cuda"), torch.zeros(P + 1, device="cuda"), held, us, **hp)


def test_empty_cases_on_device():
    p = torch.ones(16, device="cuda")
    v = torch.ones(16, device="cuda")
    rows = [torch.ones(16, device="cuda")]
    star.star_group_update(p, v, rows, star.UpdateStream([0], []), lr=0.1, momentum_coef=0.9, **opts())
    torch.cuda.synchronize()
    assert torch.all(p == 1) and torch.all(v == 1)
    n = torch.full((2,), 5.0, device="cuda")
    e = torch.empty(0, device="cuda")
    star.star_group_update(e, e, [e], star.UpdateStream([0, 1, 2], [0, 0]), lr=0.1, momentum_coef=0.9, norms_out=n,
                           **opts())
    torch.cuda.synchronize()
    assert n.tolist() == [0.0, 0.0]


def test_non_default_stream_and_back_to_back_calls():
    """Four calls enqueued without a host sync on a side stream, state carried
    from call to call (how a streamed batch of updates arrives)."""
    rng = np.random.default_rng(13)
    W, P, U = 16, 100003, 16
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    ep, ev = p0.copy(), np.zeros(P, np.float32)
    s = torch.cuda.Stream()
    p = torch.from_numpy(p0).cuda()
    v = torch.zeros(P, device="cuda")
    sets, streams, norms = [], [], []
    for call in range(4):
        rows = rand_rows(rng, W, P, "bf16", std=5e-4)
        offs, mem, st = rand_stream(rng, W, U, min_y=2, stale=8)
        sets.append((rows, to_dev_rows(rows)))
        streams.append((offs, mem, st))
        norms.append(torch.zeros(U, device="cuda"))
    torch.cuda.synchronize()
    hp = dict(lr=0.01, momentum_coef=0.9, weight_decay=1e-4, wmode="stale")
    for call in range(4):
        offs, mem, st = streams[call]
        star.star_group_update(p, v, sets[call][1], star.UpdateStream(offs, mem, st), norms_out=norms[call],
                               stream=s, **opts(), **hp)
    s.synchronize()
    for call in range(4):
        offs, mem, st = streams[call]
        ep, ev, en = so.group_update(ep, ev, sets[call][0], offs, mem, staleness=st, want_norms=True, **hp)
        np.testing.assert_allclose(norms[call].cpu().numpy(), en, rtol=TOL["bf16"])
    check(p.cpu().numpy(), v.cpu().numpy(), None, ep, ev, None, "bf16", "4 streamed calls")


def test_selector_groups_drive_the_update():
    """Iteration times -> STAR-H groups (dynamic x-order here) -> one round of
    updates with the rate scaled by the group size, against the oracle."""
    rng = np.random.default_rng(14)
    T = [0.30, 0.31, 0.33, 0.52, 0.55, 0.90, 0.29, 0.32]
    r = star.star_select_mode_ps(T, 4000.0, 1024.0)
    assert r["mode"] == star.MODE_DYNAMIC_X and len(r["groups"]) == 3
    W, P = len(T), 30011
    rows = rand_rows(rng, W, P, "f32")
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=0.1, momentum_coef=0.9, weight_decay=1e-4, scale_lr_by_group=True, want_norms=True)
    ep, ev, en = so.group_update(p0, v0, rows, r["offsets"], r["members"], **hp)
    for kern in (star.KERNEL_SEQ, star.KERNEL_AFFINE):
        p, v, n = gpu_update(p0, v0, rows, r["offsets"], r["members"], kernel=kern, **hp)
        check(p, v, n, ep, ev, en, "f32", f"selector kern={kern}")


def test_concurrent_host_threads_on_their_own_streams():
    """Four host threads, each with its own stream and shard, call the library at
    the same time; every result must equal the single-threaded one bit for bit."""
    import threading
    rng = np.random.default_rng(15)
    W, P, U = 8, 200003, 12
    jobs = []
    for t in range(4):
        rows = rand_rows(rng, W, P, "f32")
        offs, mem, st = rand_stream(rng, W, U, stale=3)
        p0 = rng.standard_normal(P).astype(np.float32)
        jobs.append((rows, to_dev_rows(rows), offs, mem, st, p0))
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")

    call_opts = opts()      # read here: the worker threads below must not depend on the fixture's state

    def run_one(job, stream, out):
        rows, drows, offs, mem, st, p0 = job
        p = torch.from_numpy(p0).cuda()
        v = torch.zeros(P, device="cuda")
        n = torch.zeros(U, device="cuda")
        torch.cuda.synchronize()
        for _ in range(5):                       # several calls, so that the threads really overlap
            star.star_group_update(p, v, drows, star.UpdateStream(offs, mem, st), norms_out=n, stream=stream, **call_opts, **hp)
        stream.synchronize()
        out.append((p.cpu().numpy(), v.cpu().numpy(), n.cpu().numpy()))

    serial = []
    for job in jobs:
        o = []
        run_one(job, torch.cuda.Stream(), o)
        serial.append(o[0])
    results = [[] for _ in jobs]
    threads = [threading.Thread(target=run_one, args=(job, torch.cuda.Stream(), results[i])) for i, job in enumerate(jobs)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for s, r in zip(serial, results):
        for a, b in zip(s, r[0]):
            assert np.array_equal(a, b)


def test_very_long_stream():
    """Thousands of updates in one call: the collapsed route composes them on the host."""
    rng = np.random.default_rng(16)
    W, P, U = 6, 4099, 5000
    rows = rand_rows(rng, W, P, "f32", std=1e-3)
    offs, mem, _ = rand_stream(rng, W, U)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=1e-3, momentum_coef=0.9, weight_decay=1e-4, want_norms=True)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, **hp)
    p, v, n = gpu_update(p0, v0, rows, offs, mem, **hp)
    check(p, v, n, ep, ev, en, "f32", "U=5000")


def test_interleaved_shards_shapes_and_kernels_without_host_sync():
    """24 calls on two streams, cycling through three shards of different length, row count, dtype and
    update count (so that consecutive launches differ in kernel, grid size and workgroup size), with no
    host synchronisation in between.  Every shard's final state and last norms must match the oracle
    applied to the same sequence: the workspace slots and their work queues are reused many times."""
    rng = np.random.default_rng(2024)
    specs = [(16, 200003, "f32", 9), (28, 150001, "bf16", 5), (6, 333337, "f32", 1)]
    shards = []
    for W, P, dtype, U in specs:
        rows = rand_rows(rng, W, P, dtype)
        p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
        shards.append(dict(W=W, P=P, dtype=dtype, U=U, rows=rows, dev=to_dev_rows(rows),
                           p=torch.from_numpy(p0).cuda(), v=torch.zeros(P, device="cuda"), ep=p0, ev=np.zeros(P, np.float32),
                           n=torch.zeros(U, device="cuda"), en=None))
    hp = dict(lr=0.02, momentum_coef=0.9, weight_decay=1e-4, wmode="stale")
    s = [torch.cuda.Stream(), torch.cuda.Stream()]
    calls = []
    for k in range(24):
        sh = shards[k % 3]
        offs, mem, st = rand_stream(rng, sh["W"], sh["U"], stale=3)
        calls.append((k % 3, offs, mem, st))
    torch.cuda.synchronize()
    for k, (i, offs, mem, st) in enumerate(calls):
        sh = shards[i]
        # a shard always uses the same stream, so its calls stay ordered; the two streams overlap
        star.star_group_update(sh["p"], sh["v"], sh["dev"], star.UpdateStream(offs, mem, st), norms_out=sh["n"],
                               stream=s[i % 2], **opts(), **hp)
    for x in s:
        x.synchronize()
    for i, offs, mem, st in calls:
        sh = shards[i]
        sh["ep"], sh["ev"], sh["en"] = so.group_update(sh["ep"], sh["ev"], sh["rows"], offs, mem, staleness=st,
                                                      want_norms=True, **hp)
    for sh in shards:
        check(sh["p"].cpu().numpy(), sh["v"].cpu().numpy(), sh["n"].cpu().numpy(), sh["ep"], sh["ev"], sh["en"],
              sh["dtype"], f"interleaved W={sh['W']} {sh['dtype']}")
