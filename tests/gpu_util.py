"""Shared helpers of the GPU parity tests: move host inputs to the device, call
the library through its binding, bring results back."""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star

TOL = {"f32": 1e-6, "bf16": 4e-3}   # max |x-ref| / (|ref| + RMS(ref)), per gradient dtype
# Both sides read a bf16 row as the same bits and compute in fp32 / fp64 from there, so the bf16 cases in fact
# hold a bound of the fp32 kind; the parity checks assert it besides the stated one.
TOL_BF16_OBSERVED = 3e-6


_TILE_ORDER = {"queue_threshold": None}


@pytest.fixture(autouse=True, params=["fixed", "queue"])
def tile_order(request):
    """Runs every test of a module that imports it twice: with the fixed assignment of tiles to
    workgroups and with tiles claimed from the work queue (which the library itself only uses
    from 16 Mi elements on), so that the small, fully checked cases cover both.  The tests pass
    the setting to every call as a per-call option: ``**opts()``."""
    _TILE_ORDER["queue_threshold"] = 1 if request.param == "queue" else 1 << 62
    yield request.param
    _TILE_ORDER["queue_threshold"] = None


def opts(kernel=None):
    """Per-call options of the running test: the fixture's tile order and, if given, a forced kernel."""
    d = dict(_TILE_ORDER)
    if kernel is not None:
        d["kernel"] = kernel
    return d


def to_dev_rows(rows_np):
    out = []
    for r in rows_np:
        if r is None:
            out.append(None)
        elif r.dtype == np.uint16:
            out.append(torch.from_numpy(r.view(np.int16).copy()).cuda().view(torch.bfloat16))
        else:
            out.append(torch.from_numpy(r.copy()).cuda())
    return out


def rand_stream(rng, W, U, min_y=1, max_y=None, stale=None):
    max_y = max_y or W
    offs, mem = [0], []
    for _ in range(U):
        y = int(rng.integers(min_y, max_y + 1))
        mem += [int(x) for x in rng.permutation(W)[:y]]
        offs.append(len(mem))
    st = None if stale is None else rng.integers(0, stale + 1, size=len(mem)).astype(np.int32)
    return np.array(offs, np.int32), np.array(mem, np.int32), st


def rand_rows(rng, W, P, dtype, std=1e-2):
    rows = []
    for _ in range(W):
        x = (rng.standard_normal(P) * std).astype(np.float32)
        if dtype == "bf16":
            x = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        rows.append(x)
    return rows


def gpu_update(p0, v0, rows_np, offs, mem, *, kernel=star.KERNEL_AUTO, want_norms=False, staleness=None, coeff=None,
               lr_per_update=None, dev_rows=None, **hp):
    """Runs star_group_update on copies of p0, v0; returns numpy (p, v, norms)."""
    p = torch.from_numpy(np.array(p0, dtype=np.float32)).cuda()
    v = torch.from_numpy(np.array(v0, dtype=np.float32)).cuda()
    rows = dev_rows if dev_rows is not None else to_dev_rows(rows_np)
    us = star.UpdateStream(offs, mem, staleness, coeff, lr_per_update)
    norms = torch.full((max(us.U, 1),), -1.0, dtype=torch.float32, device="cuda") if want_norms else None
    star.star_group_update(p, v, rows, us, norms_out=norms, **opts(kernel), **hp)
    torch.cuda.synchronize()
    return p.cpu().numpy(), v.cpu().numpy(), (None if norms is None else norms.cpu().numpy()[:us.U])
