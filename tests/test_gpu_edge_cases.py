"""GPU parity on the degenerate inputs the header makes promises about: non-finite gradients, gradient
rows that alias each other, group averages that nearly cancel, and per-call options used by several
host threads at once."""
import threading

import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
from oracle import star_oracle as so
from gpu_util import TOL, gpu_update, opts, rand_rows, rand_stream, tile_order, to_dev_rows  # noqa: F401 (tile_order: autouse fixture)

pytestmark = pytest.mark.gpu

KERNELS = {"auto": None, "seq": star.KERNEL_SEQ, "affine": star.KERNEL_AFFINE, "mfma": star.KERNEL_AFFINE_MFMA}


def masked_err(x, ref):
    """max_rel_err over the elements that are finite in the reference."""
    m = np.isfinite(ref)
    return so.max_rel_err(np.asarray(x)[m], np.asarray(ref)[m]) if m.any() else 0.0


@pytest.mark.parametrize("kname", ["seq", "affine", "mfma", "auto"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_non_finite_gradients_propagate_like_the_oracle(kname, dtype):
    """+inf, -inf and NaN at known positions of two workers' rows.  Params and momentum are non-finite
    exactly where the oracle's are; the norm of a group is non-finite exactly when the group contains
    one of the two workers; everything else matches to the usual tolerance.  A third worker that no
    group references holds NaN everywhere and must not matter."""
    rng = np.random.default_rng(41)
    W, P, U = 7, 9001, 9
    rows32 = [(rng.standard_normal(P) * 1e-2).astype(np.float32) for _ in range(W)]
    rows32[2][[5, 1024, 4097]] = [np.inf, -np.inf, np.nan]
    rows32[4][[5, 7000, P - 1]] = [-np.inf, np.inf, np.nan]      # element 5: +inf and -inf meet in groups with both
    rows32[6][:] = np.nan                                       # never referenced
    if dtype == "bf16":
        rows = [torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy() for r in rows32]
    else:
        rows = rows32
    # groups over workers 0..5: some with worker 2, some with 4, some with both, some with neither
    groups = [[0, 1], [2], [0, 4, 5], [2, 4], [1, 3, 5], [0, 1, 2, 3, 4, 5], [3], [4, 0], [5, 1, 3]]
    offs = np.cumsum([0] + [len(g) for g in groups]).astype(np.int32)
    mem = np.concatenate(groups).astype(np.int32)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3)
    with np.errstate(all="ignore"):
        ep, ev, en = so.group_update(p0, v0, rows, offs, mem, want_norms=True, **hp)
    p, v, n = gpu_update(p0, v0, rows, offs, mem, want_norms=True, kernel=KERNELS[kname], **hp)
    assert np.array_equal(np.isfinite(p), np.isfinite(ep)), "params: finiteness differs from the oracle"
    assert np.array_equal(np.isfinite(v), np.isfinite(ev)), "momentum: finiteness differs from the oracle"
    assert int((~np.isfinite(ep)).sum()) == 5               # elements 5, 1024, 4097, 7000, P-1 and no other
    tol = TOL[dtype]
    assert masked_err(p, ep) <= tol and masked_err(v, ev) <= tol
    bad = np.array([bool({2, 4} & set(g)) for g in groups])
    assert np.array_equal(~np.isfinite(en), bad)            # the oracle itself: bad exactly for those groups
    assert np.array_equal(~np.isfinite(n), bad), (kname, n)
    good = ~bad
    assert np.max(np.abs(n[good] - en[good]) / en[good]) <= tol


@pytest.mark.parametrize("kname", ["seq", "affine", "mfma", "auto"])
def test_gradient_rows_may_alias_each_other(kname):
    """Several entries of grad_rows point at the same buffer (two workers reporting the same gradient)."""
    rng = np.random.default_rng(42)
    W, P, U = 6, 70001, 8
    base = rand_rows(rng, 3, P, "f32")
    which = [0, 1, 0, 2, 1, 0]                               # worker -> buffer
    rows = [base[k] for k in which]
    dev_base = to_dev_rows(base)
    dev_rows = [dev_base[k] for k in which]
    assert dev_rows[0].data_ptr() == dev_rows[2].data_ptr() == dev_rows[5].data_ptr()
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = np.zeros(P, np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, staleness=st, want_norms=True, **hp)
    p, v, n = gpu_update(p0, v0, None, offs, mem, staleness=st, want_norms=True, kernel=KERNELS[kname],
                         dev_rows=dev_rows, **hp)
    assert so.max_rel_err(p, ep) <= 1e-6 and so.max_rel_err(v, ev) <= 1e-6
    assert np.max(np.abs(n - en) / en) <= 1e-6
    # aggregation and Gram matrix on the same aliased rows
    outs = [torch.zeros(P, device="cuda") for _ in range(U)]
    star.star_group_reduce(outs, dev_rows, star.UpdateStream(offs, mem, st), wmode="stale", **opts())
    g = torch.zeros((W, W), dtype=torch.float64, device="cuda")
    star.star_group_gram(dev_rows, g, **opts())
    torch.cuda.synchronize()
    eo = so.group_reduce(rows, offs, mem, wmode="stale", staleness=st)
    assert max(so.max_rel_err(outs[u].cpu().numpy(), eo[u]) for u in range(U)) <= 1e-6
    eg = so.gram(rows)
    assert np.max(np.abs(g.cpu().numpy() - eg) / np.sqrt(np.outer(np.diag(eg), np.diag(eg)))) <= 1e-6


def condition(rows32, offs, mem, coef):
    """kappa_u = (sum_w |c_w| ||g_w||)^2 / ||sum_w c_w g_w||^2 of every group, from float64 copies of the rows."""
    R = [np.asarray(r, np.float64) for r in rows32]
    out = []
    for u in range(len(offs) - 1):
        ids, c = mem[offs[u]:offs[u + 1]], coef[offs[u]:offs[u + 1]]
        gbar = sum(cw * R[w] for w, cw in zip(ids, c))
        out.append(sum(abs(cw) * np.linalg.norm(R[w]) for w, cw in zip(ids, c)) ** 2 / float(gbar @ gbar))
    return np.array(out)


@pytest.mark.parametrize("times", [1, 4])
def test_signed_coefficients_take_the_direct_norm_route(times):
    """Caller-given coefficients of both signs on nearly identical rows: the group 'average' is a small
    difference of large rows.  The library takes such norms from the direct sums of gbar^2 (not from the
    Gram matrix, whose quadratic form would cancel), and they hold the ordinary tolerance.  The stream of
    three updates is short enough for the literal kernel (direct sums in the same pass); four times over it
    takes the collapsed update with a direct norm pass beside it."""
    rng = np.random.default_rng(43)
    W, P = 4, 300007
    g = (rng.standard_normal(P) * 1e-2).astype(np.float32)
    rows = [(g + (rng.standard_normal(P) * 1e-5).astype(np.float32)) for _ in range(W)]
    offs = np.concatenate([[0], np.cumsum(np.tile([2, 2, 4], times))]).astype(np.int32)
    mem = np.tile(np.array([0, 1, 2, 3, 0, 1, 2, 3], np.int32), times)
    cf = np.tile(np.array([1, -1, 0.5, -0.5, 1, -1, 1, -1], np.float32), times)
    us = star.UpdateStream(offs, mem, None, cf)
    c = star.star_plan_choice(P, W, "f32", us, lr=0.1, momentum_coef=0.9, wmode="explicit", want_norms=True)
    if times == 1:
        assert c["kernel"] == star.KERNEL_SEQ and c["launches"] == 1 and c["collapsed_update"] == 0
    else:
        assert c["kernel"] == star.KERNEL_AFFINE and c["launches"] == 2      # collapsed update + one direct norm pass
    kappa = condition(rows, offs, mem, cf)
    assert kappa.min() > 1e5                                            # the quadratic form would lose 5 digits
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)   # momentum on the scale of the rows: the state is judged
    hp = dict(lr=0.1, momentum_coef=0.9, weight_decay=1e-4, wmode="explicit")   # against that scale, the norms on their own
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, coeff=cf, want_norms=True, **hp)
    p, v, n = gpu_update(p0, v0, rows, offs, mem, coeff=cf, want_norms=True, **hp)
    e_n = float(np.max(np.abs(n - en) / en))
    print(f"signed coefficients: kappa {kappa.min():.3g}..{kappa.max():.3g}, norm err {e_n:.3g}", flush=True)
    # (twelve updates let the initial momentum decay to a quarter, and what is left of v is then mostly the
    # cancelling sum of the rows, whose terms are a thousand times the result: the fp32 coefficients' own
    # rounding shows at 4e-6 of it; the norms have no such excuse)
    tol = 1e-6 if times == 1 else 1e-5
    assert so.max_rel_err(p, ep) <= tol and so.max_rel_err(v, ev) <= tol and e_n <= 1e-6
    # norms alone take the same route
    n2 = torch.zeros(3 * times, device="cuda")
    star.star_group_norms(to_dev_rows(rows), us, n2, wmode="explicit", **opts())
    torch.cuda.synchronize()
    assert np.max(np.abs(n2.cpu().numpy() - en) / en) <= 1e-6


@pytest.mark.parametrize("kname", ["affine", "mfma", "auto", "seq"])
def test_anticorrelated_rows_hold_the_documented_norm_bound(kname):
    """g_1 = -g_0 + small noise under plain mean weights: the group average nearly cancels although every
    coefficient is positive.  The header's bound for norms that come from the Gram matrix: relative error
    at most 2e-8 * kappa_u (kappa_u as computed above; 1..y_u for ordinary groups).  The direct route
    (seq) is not subject to it and holds 1e-6."""
    rng = np.random.default_rng(44)
    W, P = 4, 200003
    g0 = (rng.standard_normal(P) * 1e-2).astype(np.float32)
    rows = [g0, (-g0 + (rng.standard_normal(P) * 1e-4).astype(np.float32)),
            (rng.standard_normal(P) * 1e-2).astype(np.float32), (rng.standard_normal(P) * 1e-2).astype(np.float32)]
    offs = np.array([0, 2, 4, 8], np.int32)
    mem = np.array([0, 1, 2, 3, 0, 1, 2, 3], np.int32)
    coef = np.concatenate([np.full(2, 0.5), np.full(2, 0.5), np.full(4, 0.25)])
    kappa = condition(rows, offs, mem, coef)
    en = so.group_norms(rows, offs, mem)
    n = torch.zeros(3, device="cuda")
    star.star_group_norms(to_dev_rows(rows), star.UpdateStream(offs, mem), n, **opts(KERNELS[kname]))
    torch.cuda.synchronize()
    err = np.abs(n.cpu().numpy() - en) / en
    print(f"anti-correlated rows {kname}: kappa {np.round(kappa, 1).tolist()}, norm err {err.tolist()}", flush=True)
    assert kappa[0] > 1e4 and kappa[1] < 4
    if kname == "seq":
        assert err.max() <= 1e-6
    else:
        assert np.all(err <= 2e-8 * kappa)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_direct_norms_option_on_anticorrelated_rows(dt):
    """The same kind of rows with STAR_OPT_DIRECT_NORMS: the update is still the collapsed one, the
    norms come from direct sums in a pass of their own and hold 1e-6 on the cancelling group too, where
    the Gram route of the same call without the flag is allowed 2e-8 * kappa."""
    rng = np.random.default_rng(46)
    W, P = 8, 300011
    rows = rand_rows(rng, W, P, dt)
    as_f = (lambda r: r) if dt == "f32" else (lambda r: (r.astype(np.uint32) << 16).view(np.float32))
    noise = (rng.standard_normal(P) * 1e-4).astype(np.float32)
    mirror = -as_f(rows[0]) + noise
    if dt == "bf16":                      # round to nearest even onto bf16 bit patterns
        b = mirror.view(np.uint32)
        mirror = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    rows[1] = mirror
    # the four groups twice over: eight updates, too long a stream for the literal kernel (whose norms are direct anyway)
    offs = np.array([0, 2, 4, 8, 16, 18, 20, 24, 32], np.int32)
    mem = np.tile(np.array([0, 1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3, 4, 5, 6, 7], np.int32), 2)
    us = star.UpdateStream(offs, mem)
    coef = np.tile(np.concatenate([np.full(2, 0.5), np.full(2, 0.5), np.full(4, 0.25), np.full(8, 0.125)]), 2)
    kappa = condition([as_f(r) for r in rows], offs, mem, coef)
    assert kappa[0] > 1e3
    c = star.star_plan_choice(P, W, dt, us, lr=0.1, momentum_coef=0.9, weight_decay=1e-4, want_norms=True)
    assert c["kernel"] != star.KERNEL_SEQ
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)
    hp = dict(lr=0.1, momentum_coef=0.9, weight_decay=1e-4)
    ep, ev, en = so.group_update(p0, v0, rows, offs, mem, want_norms=True, **hp)
    drows = to_dev_rows(rows)
    out = {}
    for direct in (False, True):
        p, v = torch.from_numpy(p0).cuda(), torch.from_numpy(v0).cuda()
        n = torch.full((8,), -1.0, device="cuda")
        star.star_group_update(p, v, drows, us, norms_out=n, direct_norms=direct, **opts(), **hp)
        torch.cuda.synchronize()
        out[direct] = (p.cpu().numpy(), v.cpu().numpy(), np.abs(n.cpu().numpy() - en) / en)
    print(f"direct norms {dt}: kappa {np.round(kappa, 1).tolist()}, err gram {out[False][2].tolist()}, "
          f"direct {out[True][2].tolist()}", flush=True)
    assert np.all(out[False][2] <= 2e-8 * kappa + 1e-6)
    assert out[True][2].max() <= 1e-6
    for direct in (False, True):
        assert so.max_rel_err(out[direct][0], ep) <= 1e-6 and so.max_rel_err(out[direct][1], ev) <= 1e-6
    # norms alone
    n = torch.zeros(8, device="cuda")
    star.star_group_norms(drows, us, n, direct_norms=True, **opts())
    torch.cuda.synchronize()
    assert np.max(np.abs(n.cpu().numpy() - en) / en) <= 1e-6


@pytest.mark.parametrize("dt,W,norms", [("f32", 16, True), ("bf16", 16, True), ("f32", 8, False), ("f32", 24, True)])
def test_unaligned_buffers_keep_the_whole_grid(dt, W, norms):
    """Views that start one element into their allocations are not 16-byte aligned and go through the
    one-element-per-lane path.  That path is slower than the vector one but must stay within a small factor
    of it (a launch that hands the whole shard to a single workgroup is hundreds of times slower), and its
    results are the same as those of the aligned call on the same values."""
    import time
    rng = np.random.default_rng(47)
    P = 4 << 20
    big = [torch.from_numpy((rng.standard_normal(P + 8) * 1e-2).astype(np.float32)).cuda() for _ in range(W)]
    if dt == "bf16":
        big = [r.to(torch.bfloat16) for r in big]
    offs, mem, st = rand_stream(rng, W, 8, stale=3)
    us = star.UpdateStream(offs, mem, st)
    p0 = torch.from_numpy((rng.standard_normal(P + 8) * 0.02).astype(np.float32)).cuda()
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    took, outs = [], []
    for off in (0, 1):
        rows = [r[off:off + P] for r in big] if off else [r[1:1 + P].clone() for r in big]   # same values, aligned copies
        pbuf, vbuf = p0.clone(), torch.zeros(P + 8, device="cuda")
        p, v = (pbuf[1:1 + P], vbuf[1:1 + P]) if off else (pbuf[1:1 + P].clone(), vbuf[1:1 + P].clone())
        assert (p.data_ptr() % 16 != 0) == bool(off)
        n = torch.zeros(us.U, device="cuda") if norms else None
        star.star_group_update(p, v, rows, us, norms_out=n, **opts(), **hp)      # warm-up; also the result compared below
        torch.cuda.synchronize()
        outs.append((p.clone(), v.clone(), None if n is None else n.clone()))
        t0 = time.perf_counter()
        for _ in range(5):
            star.star_group_update(p, v, rows, us, norms_out=n, **opts(), **hp)
        torch.cuda.synchronize()
        took.append((time.perf_counter() - t0) / 5)
    print(f"unaligned {dt} W={W} norms={norms}: aligned {took[0] * 1e6:.0f} us, one element off {took[1] * 1e6:.0f} us", flush=True)
    assert took[1] <= 8 * took[0] + 200e-6
    a, b = outs
    assert so.max_rel_err(b[0].cpu().numpy(), a[0].cpu().numpy()) <= 2e-6
    assert so.max_rel_err(b[1].cpu().numpy(), a[1].cpu().numpy()) <= 2e-6
    if norms:
        assert np.max(np.abs(b[2].cpu().numpy() - a[2].cpu().numpy()) / a[2].cpu().numpy()) <= 2e-6


def test_two_threads_with_different_options():
    """Two host threads call the library at the same time with different per-call options (one forces
    the step-by-step kernel and the queue, the other the collapsed kernel and the fixed assignment);
    each must get exactly what it gets alone: there is no process-wide setting to trample on."""
    rng = np.random.default_rng(45)
    W, P, U = 8, 300007, 6
    rows = rand_rows(rng, W, P, "f32")
    drows = to_dev_rows(rows)
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    settings = [dict(kernel=star.KERNEL_SEQ, queue_threshold=1), dict(kernel=star.KERNEL_AFFINE, queue_threshold=1 << 62)]

    def run_one(o, out, reps):
        stream = torch.cuda.Stream()
        p = torch.from_numpy(p0).cuda()
        v = torch.zeros(P, device="cuda")
        n = torch.zeros(U, device="cuda")
        torch.cuda.synchronize()
        for _ in range(reps):
            star.star_group_update(p, v, drows, star.UpdateStream(offs, mem, st), norms_out=n, stream=stream, **o, **hp)
        stream.synchronize()
        out.append((p.cpu().numpy(), v.cpu().numpy(), n.cpu().numpy()))

    alone = []
    for o in settings:
        r = []
        run_one(o, r, 8)
        alone.append(r[0])
    assert not np.array_equal(alone[0][0], alone[1][0])      # the two evaluations round differently: the options matter
    together = [[], []]
    threads = [threading.Thread(target=run_one, args=(o, together[i], 8)) for i, o in enumerate(settings)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for a, b in zip(alone, together):
        for x, y in zip(a, b[0]):
            assert np.array_equal(x, y)
