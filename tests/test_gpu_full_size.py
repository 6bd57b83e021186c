"""Parity at the five workloads' full sizes, in the configuration bench.py times.

The oracle cannot run 1e8 elements x 64 updates in test time, but every element
is independent, so the updated state is checked on sampled elements (head, the
ragged tail, windows at odd offsets): the oracle is run on exactly those
elements.  Norms couple all elements; they are checked (a) against the oracle
over the full shard for the two smallest groups of the call, and (b) for every
update against the library's other, independent norm route (direct sum of
squares versus pairwise products), which must agree far inside the tolerance.
"""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
import workloads
from oracle import star_oracle as so
from gpu_util import TOL

pytestmark = pytest.mark.gpu


def sample_indices(P, rng, window=2048, n_mid=6):
    parts = [np.arange(0, min(window, P)), np.arange(max(0, P - window - 3), P)]
    for _ in range(n_mid):
        lo = int(rng.integers(0, max(1, P - window))) | 1          # odd offsets: not chunk aligned
        parts.append(np.arange(lo, min(P, lo + window)))
    return np.unique(np.concatenate(parts))


def rows_at(rows, idx_dev):
    out = []
    for r in rows:
        x = r[idx_dev].cpu()
        out.append(x.view(torch.int16).numpy().view(np.uint16).copy() if x.dtype == torch.bfloat16 else x.numpy())
    return out


@pytest.mark.parametrize("name", workloads.ORDER)
def test_full_size_workload(name):
    wl = workloads.WORKLOADS[name]
    print(f"full-size {name}: P={wl.P} W={wl.W} U={wl.U}x{wl.calls} {wl.grad_dtype}", flush=True)
    rng = np.random.default_rng(123)
    idx = sample_indices(wl.P, rng)
    idx_dev = torch.from_numpy(idx).cuda()
    p = workloads.make_params(wl, 0, "cuda")
    v = workloads.make_momentum(wl, "cuda")
    ep, ev = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    hp = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay, wmode=wl.wmode)
    tol = TOL[wl.grad_dtype]
    rows = None
    for call in range(wl.calls):
        if rows is None or wl.fresh_grads_per_call:
            rows = None                                     # free the previous set first
            rows = workloads.make_grad_rows(wl, 0, call, "cuda")
        s = workloads.make_update_stream(wl, 0, call)
        us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
        norms = torch.zeros(wl.U, device="cuda")            # asked for on every workload here
        star.star_group_update(p, v, rows, us, norms_out=norms, **hp)
        torch.cuda.synchronize()
        # state on the sampled elements
        ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), s["offsets"], s["members"],
                                    staleness=s["staleness"], **hp)
        e_p = so.max_rel_err(p[idx_dev].cpu().numpy(), ep)
        e_v = so.max_rel_err(v[idx_dev].cpu().numpy(), ev)
        print(f"  call {call}: sampled {idx.size} elements, err params {e_p:.3g} momentum {e_v:.3g}", flush=True)
        assert e_p <= tol and e_v <= tol
        # norms: second route on the GPU for all updates
        n_gpu = norms.cpu().numpy()
        star.star_set_kernel(star.KERNEL_SEQ)
        try:
            norms2 = torch.zeros(wl.U, device="cuda")
            star.star_group_norms(rows, us, norms2, wmode=wl.wmode)
            torch.cuda.synchronize()
        finally:
            star.star_set_kernel(star.KERNEL_AUTO)
        e_routes = float(np.max(np.abs(n_gpu - norms2.cpu().numpy()) / norms2.cpu().numpy()))
        # norms: oracle over the whole shard for the two smallest groups
        sizes = np.diff(s["offsets"])
        pick = np.argsort(sizes, kind="stable")[:2]
        offs, mem, st = [0], [], []
        for u in pick:
            lo, hi = s["offsets"][u], s["offsets"][u + 1]
            mem += list(s["members"][lo:hi])
            st += list(s["staleness"][lo:hi]) if s["staleness"] is not None else [0] * (hi - lo)
            offs.append(len(mem))
        need = sorted(set(mem))
        host_rows = [None] * wl.W
        for w in range(wl.W):
            if w in need:
                x = rows[w].cpu()
                host_rows[w] = (x.view(torch.int16).numpy().view(np.uint16) if x.dtype == torch.bfloat16
                                else x.numpy())
            else:                                        # never read by the oracle for these groups
                host_rows[w] = host_rows[need[0]] if host_rows[need[0]] is not None else None
        first = next(r for r in host_rows if r is not None)
        host_rows = [r if r is not None else first for r in host_rows]
        en = so.group_norms(host_rows, offs, mem, wmode=wl.wmode, staleness=st)
        e_n = float(np.max(np.abs(n_gpu[pick] - en) / en))
        print(f"  call {call}: norms vs oracle (updates {pick.tolist()}, sizes {sizes[pick].tolist()}) {e_n:.3g}; "
              f"two GPU routes differ by {e_routes:.3g}", flush=True)
        assert e_n <= tol and e_routes <= min(tol, 2e-6)
        del host_rows, norms, norms2
    del p, v, rows
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["bert_base", "vgg16"])
def test_full_size_publish_and_reduce(name):
    """The widened entry points at full workload size, on sampled elements:
    update with a bf16 copy of the new parameters, and one full-group
    aggregation with bf16 output."""
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
    tol = TOL[wl.grad_dtype]
    assert so.max_rel_err(p[idx_dev].cpu().numpy(), ep) <= tol
    assert torch.equal(pub[idx_dev].cpu(), p[idx_dev].cpu().to(torch.bfloat16))
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
    # the norm against the Gram matrix of the rows where that is built (W <= 16), else against the output itself
    if wl.W <= 16:
        g = torch.zeros((wl.W, wl.W), dtype=torch.float64, device="cuda")
        star.star_group_gram(rows, g)
        torch.cuda.synchronize()
        ref = float(torch.sqrt(g.sum()).item()) / wl.W
    else:
        ref = float(torch.linalg.vector_norm(out[0].float().double()).item())
    assert abs(n.item() / ref - 1) <= (1e-5 if wl.W <= 16 else 2e-3)


@pytest.mark.parametrize("name", ["bert_base", "bert_large"])
def test_full_size_single_update(name):
    """One update per call at full size (every gradient report applied on arrival): fp32 rows take the
    step-by-step kernel in queue order, bf16 rows the collapsed one.  State on sampled elements, the
    one norm against the oracle over the whole shard."""
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
    tol = TOL[wl.grad_dtype]
    ep, ev = p[idx_dev].cpu().numpy(), v[idx_dev].cpu().numpy()
    norms = torch.zeros(1, device="cuda")
    for call in range(2):                                   # twice: the second call starts from the first's state
        star.star_group_update(p, v, rows, star.UpdateStream(offs, mem, st), norms_out=norms, **hp)
        torch.cuda.synchronize()
        ep, ev, _ = so.group_update(ep, ev, rows_at(rows, idx_dev), offs, mem, staleness=st, **hp)
        assert so.max_rel_err(p[idx_dev].cpu().numpy(), ep) <= tol
        assert so.max_rel_err(v[idx_dev].cpu().numpy(), ev) <= tol
    host_rows = []
    first = None
    for w in range(wl.W):
        if w in set(int(m) for m in mem):
            x = rows[w].cpu()
            host_rows.append(x.view(torch.int16).numpy().view(np.uint16) if x.dtype == torch.bfloat16 else x.numpy())
            first = host_rows[-1] if first is None else first
        else:
            host_rows.append(None)
    host_rows = [r if r is not None else first for r in host_rows]     # rows outside the group are never read
    en = so.group_norms(host_rows, offs, mem, wmode=wl.wmode, staleness=st)
    e_n = abs(float(norms.cpu().numpy()[0]) - float(en[0])) / float(en[0])
    print(f"  norm vs oracle over the whole shard: {e_n:.3g}", flush=True)
    assert e_n <= min(tol, 2e-6)
    del p, v, rows, host_rows
    torch.cuda.empty_cache()
