"""Parity at the five workloads' full sizes, in the configuration bench.py times.

State (params, momentum).  Every element is independent, so the oracle can be run on any subset.  The
checked subset holds one element of every block of 512 consecutive elements, at a seeded offset
inside the block, plus the first 2048 elements and the ragged tail: every tile a workgroup can claim
from the work queue (1024 elements, 512 for the half-size workgroups of the 32-row kernels) has
elements in it, so a tile that is skipped, done twice or done with another tile's rows shows up.  On
tiny and resnet50 the oracle runs over the whole array.

Norms couple all elements.  They are compared with the oracle's norms over the whole shard: every
update of tiny, resnet50 and bert_base; on vgg16 and bert_large eight updates per call, spread from
the smallest group to the largest.  The oracle is the plain single-threaded C loop; this test only
runs several instances of it side by side (one per group, or one per slice of the array).
The comparison of the library's two norm routes with each other is kept as a self-check and is
labelled so: it is no parity evidence.
"""
import concurrent.futures

import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
import workloads
from oracle import star_oracle as so
from gpu_util import TOL, TOL_BF16_OBSERVED

pytestmark = pytest.mark.gpu

BLOCK = 512
WORKERS = 16


def sample_indices(P, rng, edge=2048):
    nblock = (P + BLOCK - 1) // BLOCK
    inner = np.arange(nblock, dtype=np.int64) * BLOCK + rng.integers(0, BLOCK, size=nblock)
    inner = inner[inner < P]
    return np.unique(np.concatenate([np.arange(0, min(edge, P)), inner, np.arange(max(0, P - edge - 3), P)]))


def to_host(r):
    x = r.cpu()
    return x.view(torch.int16).numpy().view(np.uint16) if x.dtype == torch.bfloat16 else x.numpy()


def rows_at(rows, idx_dev):
    return [to_host(r[idx_dev]).copy() for r in rows]


def pmap(fn, items):
    with concurrent.futures.ThreadPoolExecutor(max_workers=WORKERS) as ex:
        return list(ex.map(fn, items))


def oracle_norms(host_rows, s, wmode, pick):
    """Oracle norms over the whole shard of the updates in `pick`, one oracle call per update."""
    def one(u):
        lo, hi = int(s["offsets"][u]), int(s["offsets"][u + 1])
        st = None if s["staleness"] is None else s["staleness"][lo:hi]
        return float(so.group_norms(host_rows, [0, hi - lo], s["members"][lo:hi], wmode=wmode, staleness=st)[0])
    return np.array(pmap(one, [int(u) for u in pick]))


def oracle_update_whole(p, v, host_rows, s, hp):
    """Oracle over the whole array, cut into contiguous slices that run side by side (elements are
    independent); the slices' squared norms add up."""
    P = p.shape[0]
    cuts = np.linspace(0, P, WORKERS + 1).astype(np.int64)

    def one(k):
        lo, hi = int(cuts[k]), int(cuts[k + 1])
        return so.group_update(p[lo:hi], v[lo:hi], [r[lo:hi] for r in host_rows], s["offsets"], s["members"],
                               staleness=s["staleness"], want_norms=True, **hp)
    parts = pmap(one, range(WORKERS))
    ep = np.concatenate([a for a, _, _ in parts])
    ev = np.concatenate([b for _, b, _ in parts])
    en = np.sqrt(np.sum(np.stack([c for _, _, c in parts]) ** 2, axis=0))
    return ep, ev, en


def spread(sizes, n):
    """n updates from the smallest group to the largest (all of them when there are no more than n)."""
    order = np.argsort(sizes, kind="stable")
    if len(order) <= n:
        return order
    return order[np.unique(np.round(np.linspace(0, len(order) - 1, n)).astype(int))]


WHOLE = ("tiny", "resnet50")          # oracle over the whole array
ALL_NORMS = ("tiny", "resnet50", "bert_base")


@pytest.mark.parametrize("name", workloads.ORDER)
def test_full_size_workload(name):
    wl = workloads.WORKLOADS[name]
    print(f"full-size {name}: P={wl.P} W={wl.W} U={wl.U}x{wl.calls} {wl.grad_dtype}", flush=True)
    rng = np.random.default_rng(123)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    whole = name in WHOLE
    ep, ev = (p.cpu().numpy(), v.cpu().numpy()) if whole else (p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy())
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    tol = min(TOL[wl.grad_dtype], TOL_BF16_OBSERVED)
    choice = None
    rows = None
    for call in range(wl.calls):
        if rows is None or wl.fresh_grads_per_call:
            rows = None                                     # free the previous set first
            rows = workloads.make_grad_rows(wl, 0, call, "cuda")
        s = workloads.make_update_stream(wl, 0, call)
        us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
        choice = star.star_plan_choice(wl.P, wl.W, wl.grad_dtype, us, want_norms=True, **hp)
        norms = torch.zeros(wl.U, device="cuda")            # asked for on every workload here
        star.star_group_update(p, v, rows, us, norms_out=norms, **hp)
        torch.cuda.synchronize()
        n_gpu = norms.cpu().numpy()
        host_rows = [to_host(r) for r in rows]
        sizes = np.diff(s["offsets"])
        if whole:
            ep, ev, en = oracle_update_whole(ep, ev, host_rows, s, hp)
            e_p = so.max_rel_err(p.cpu().numpy(), ep)
            e_v = so.max_rel_err(v.cpu().numpy(), ev)
            pick = np.arange(wl.U)
            checked = wl.P
        else:
            ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), s["offsets"], s["members"],
                                        staleness=s["staleness"], **hp)
            e_p = so.max_rel_err(p[idx_dev].cpu().numpy(), ep)
            e_v = so.max_rel_err(v[idx_dev].cpu().numpy(), ev)
            pick = np.arange(wl.U) if name in ALL_NORMS else spread(sizes, 8)
            en = oracle_norms(host_rows, s, wl.wmode, pick)
            checked = idx.size
        print(f"  call {call} (kernel {choice['kernel']}, queue order {choice['queue_order']}): {checked} elements "
              f"checked, err params {e_p:.3g} momentum {e_v:.3g}", flush=True)
        assert e_p <= tol and e_v <= tol
        e_n = float(np.max(np.abs(n_gpu[pick] - en) / en))
        print(f"  call {call}: {len(pick)} of {wl.U} norms vs the oracle over the whole shard "
              f"(group sizes {sorted(set(sizes[pick].tolist()))}): {e_n:.3g}", flush=True)
        assert e_n <= tol
        del host_rows
        # self-check, not parity: the library's other norm route (direct sums of squares against the
        # Gram matrix) on all updates
        norms2 = torch.zeros(wl.U, device="cuda")
        star.star_group_norms(rows, us, norms2, wmode=wl.wmode, kernel=star.KERNEL_SEQ)
        torch.cuda.synchronize()
        e_routes = float(np.max(np.abs(n_gpu - norms2.cpu().numpy()) / norms2.cpu().numpy()))
        print(f"  call {call}: self-check, the two norm routes of the library differ by {e_routes:.3g}", flush=True)
        assert e_routes <= min(tol, 2e-6)
        del norms, norms2
    del p, v, rows
    torch.cuda.empty_cache()


@pytest.mark.parametrize("norms", [True, False])
def test_long_shard_of_wide_fp32_rows(norms):
    """24 fp32 rows on a shard long enough for queue order (20 M elements), a shape none of the five workloads has:
    with norms the collapsed update with direct norm sums, without them the plain collapsed kernel with claims of
    two tiles.  State on one element of every block of 512, every norm against the oracle over the whole shard."""
    wl = workloads.WORKLOADS["bert_base"].scaled(20_000_003)
    import dataclasses
    wl = dataclasses.replace(wl, W=24, U=8, heavy_frac=0.0, norms=norms)
    rng = np.random.default_rng(9)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    rows = workloads.make_grad_rows(wl, 0, 0, "cuda")
    s = workloads.make_update_stream(wl, 0, 0)
    us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    c = star.star_plan_choice(wl.P, wl.W, "f32", us, want_norms=norms, **hp)
    assert c["queue_order"] == 1 and c["collapsed_update"] == 1
    assert c["kernel"] == (star.KERNEL_SEQ if norms else star.KERNEL_AFFINE)
    ep, ev = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    n = torch.zeros(wl.U, device="cuda") if norms else None
    star.star_group_update(p, v, rows, us, norms_out=n, **hp)
    torch.cuda.synchronize()
    ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), s["offsets"], s["members"], staleness=s["staleness"], **hp)
    e_p, e_v = so.max_rel_err(p[idx_dev].cpu().numpy(), ep), so.max_rel_err(v[idx_dev].cpu().numpy(), ev)
    print(f"wide fp32 rows, norms={norms}: {idx.size} elements, err params {e_p:.3g} momentum {e_v:.3g}", flush=True)
    assert e_p <= 1e-6 and e_v <= 1e-6
    if norms:
        en = oracle_norms([to_host(r) for r in rows], s, wl.wmode, np.arange(wl.U))
        e_n = float(np.max(np.abs(n.cpu().numpy() - en) / en))
        print(f"  all {wl.U} norms vs the oracle over the whole shard: {e_n:.3g}", flush=True)
        assert e_n <= 1e-6


@pytest.mark.parametrize("dt,W,P", [("bf16", 8, 6 * 1024 * 1024 + 1027), ("f32", 16, 2 * 1024 * 1024 + 5),
                                    ("bf16", 32, 12 * 1024 * 1024 + 77), ("f32", 12, 9 * 1024 * 1024 + 3)])
def test_mid_size_shards_in_the_even_split(dt, W, P):
    """Shards of 2 to 12 Mi elements, where the matrix-core kernel splits its tiles evenly over the workgroups
    (up to 8 or 16 tiles each for an update, up to 48 or 128 for the norms alone) or has just gone over to
    claims: update with norms on one element of every block of 512 plus both ends, and every norm -- of the
    update and of star_group_norms -- against the oracle over the whole shard."""
    import dataclasses
    wl = dataclasses.replace(workloads.WORKLOADS["bert_base"].scaled(P), W=W, U=12, grad_dtype=dt, heavy_frac=0.0, norms=True)
    rng = np.random.default_rng(17)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    rows = workloads.make_grad_rows(wl, 0, 0, "cuda")
    s = workloads.make_update_stream(wl, 0, 0)
    us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    c = star.star_plan_choice(wl.P, wl.W, dt, us, want_norms=True, **hp)
    assert c["kernel"] == star.KERNEL_AFFINE_MFMA and c["queue_order"] == 1
    ep, ev = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    n, n2 = torch.zeros(wl.U, device="cuda"), torch.zeros(wl.U, device="cuda")
    star.star_group_update(p, v, rows, us, norms_out=n, **hp)
    star.star_group_norms(rows, us, n2, wmode=wl.wmode, kernel=star.KERNEL_AFFINE_MFMA)
    torch.cuda.synchronize()
    ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), s["offsets"], s["members"], staleness=s["staleness"], **hp)
    e_p, e_v = so.max_rel_err(p[idx_dev].cpu().numpy(), ep), so.max_rel_err(v[idx_dev].cpu().numpy(), ev)
    en = oracle_norms([to_host(r) for r in rows], s, wl.wmode, np.arange(wl.U))
    e_n = float(np.max(np.abs(n.cpu().numpy() - en) / en))
    e_n2 = float(np.max(np.abs(n2.cpu().numpy() - en) / en))
    print(f"mid-size {dt} W={W} P={P}: {idx.size} elements, err params {e_p:.3g} momentum {e_v:.3g} norms {e_n:.3g} / alone {e_n2:.3g}",
          flush=True)
    tol = min(TOL[dt], TOL_BF16_OBSERVED)
    assert e_p <= tol and e_v <= tol and e_n <= 1e-6 and e_n2 <= 1e-6


@pytest.mark.parametrize("name", ["bert_base", "vgg16"])
def test_full_size_publish_and_reduce(name):
    """The widened entry points at full workload size, on one element of every block of 512: update with a
    bf16 copy of the new parameters, and one full-group aggregation with bf16 output and its norm
    against the oracle over the whole shard."""
    wl = workloads.WORKLOADS[name]
    print(f"full-size publish/reduce {name}: P={wl.P} W={wl.W}", flush=True)
    rng = np.random.default_rng(321)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    p0, v0 = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    rows = workloads.make_grad_rows(wl, 0, 0, "cuda")
    s = workloads.make_update_stream(wl, 0, 0)
    us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    pub = torch.zeros(wl.P, dtype=torch.bfloat16, device="cuda")
    star.star_group_update_publish(p, v, rows, us, pub, **hp)
    torch.cuda.synchronize()
    sub = rows_at(rows, idx_dev)
    ep, ev, _ = so.group_update(p0, v0, sub, s["offsets"], s["members"], staleness=s["staleness"], **hp)
    tol = min(TOL[wl.grad_dtype], TOL_BF16_OBSERVED)
    assert so.max_rel_err(p[idx_dev].cpu().numpy(), ep) <= tol
    assert so.max_rel_err(v[idx_dev].cpu().numpy(), ev) <= tol
    assert torch.equal(pub.float(), p.to(torch.bfloat16).float())       # the whole copy: RNE of the new params
    assert so.max_rel_err(pub[idx_dev].float().cpu().numpy(), ep) <= 4e-3
    del pub
    # aggregation of all W rows, bf16 out, norm on
    full_offs = np.array([0, wl.W], np.int32)
    full_mem = np.arange(wl.W, dtype=np.int32)
    out = [torch.zeros(wl.P, dtype=torch.bfloat16, device="cuda")]
    n = torch.zeros(1, device="cuda")
    star.star_group_reduce(out, rows, star.UpdateStream(full_offs, full_mem), norms_out=n)
    torch.cuda.synchronize()
    eo = so.group_reduce(sub, full_offs, full_mem)
    assert so.max_rel_err(out[0][idx_dev].float().cpu().numpy(), eo[0]) <= 4e-3
    # its norm against the oracle over the whole shard: the full group's squared norm is the sum over slices
    host_rows = [to_host(r) for r in rows]
    cuts = np.linspace(0, wl.P, WORKERS + 1).astype(np.int64)
    parts = pmap(lambda k: float(so.group_norms([r[cuts[k]:cuts[k + 1]] for r in host_rows], full_offs, full_mem)[0]),
                 range(WORKERS))
    ref = float(np.sqrt(np.sum(np.array(parts) ** 2)))
    e_n = abs(n.item() / ref - 1)
    print(f"  reduce norm vs the oracle over the whole shard: {e_n:.3g}", flush=True)
    assert e_n <= tol


@pytest.mark.parametrize("name", ["bert_base", "bert_large"])
def test_full_size_single_update(name):
    """One update per call at full size (every gradient report applied on arrival): fp32 rows take the
    step-by-step kernel in queue order, bf16 rows the collapsed one.  State on one element of every
    block of 512, the one norm against the oracle over the whole shard."""
    wl = workloads.WORKLOADS[name]
    rng = np.random.default_rng(77)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    rows = workloads.make_grad_rows(wl, 0, 0, "cuda")
    s = workloads.make_update_stream(wl, 0, 0)
    hi = int(s["offsets"][1])
    offs = np.array([0, hi], np.int32)
    mem = np.asarray(s["members"][:hi], np.int32)
    st = None if s["staleness"] is None else np.asarray(s["staleness"][:hi], np.int32)
    print(f"full-size single update {name}: P={wl.P} group of {hi} of {wl.W} workers", flush=True)
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    tol = min(TOL[wl.grad_dtype], TOL_BF16_OBSERVED)
    ep, ev = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    norms = torch.zeros(1, device="cuda")
    for call in range(2):                                   # twice: the second call starts from the first's state
        star.star_group_update(p, v, rows, star.UpdateStream(offs, mem, st), norms_out=norms, **hp)
        torch.cuda.synchronize()
        ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), offs, mem, staleness=st, **hp)
        assert so.max_rel_err(p[idx_dev].cpu().numpy(), ep) <= tol
        assert so.max_rel_err(v[idx_dev].cpu().numpy(), ev) <= tol
    members = set(int(m) for m in mem)
    first = to_host(rows[int(mem[0])])
    host_rows = [to_host(rows[w]) if w in members else first for w in range(wl.W)]   # rows outside the group are never read
    en = oracle_norms(host_rows, {"offsets": offs, "members": mem, "staleness": st}, wl.wmode, [0])
    e_n = abs(float(norms.cpu().numpy()[0]) - float(en[0])) / float(en[0])
    print(f"  norm vs oracle over the whole shard: {e_n:.3g}", flush=True)
    assert e_n <= min(tol, 2e-6)
    del p, v, rows, host_rows
    torch.cuda.empty_cache()
