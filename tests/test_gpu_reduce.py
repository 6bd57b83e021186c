"""GPU parity of star_group_reduce (aggregation without the optimizer step)
against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
from oracle import star_oracle as so
from gpu_util import TOL, opts, rand_rows, rand_stream, tile_order, to_dev_rows  # noqa: F401 (tile_order: autouse fixture)

pytestmark = pytest.mark.gpu


def run_reduce(rows_np, offs, mem, st, out_dtype, norms, P, wmode="stale", shift=0):
    drows = to_dev_rows(rows_np)
    U = len(offs) - 1
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    backing = [torch.full((P + 8,), 7.0, dtype=tdt, device="cuda") for _ in range(U)]
    outs = [b[shift:shift + P] for b in backing]
    n = torch.full((max(U, 1),), -1.0, device="cuda") if norms else None
    star.star_group_reduce(outs, drows, star.UpdateStream(offs, mem, st), wmode=wmode, norms_out=n, **opts())
    torch.cuda.synchronize()
    for b in backing:                                   # nothing written outside [shift, shift+P)
        assert torch.all(b[:shift] == 7.0) and torch.all(b[shift + P:] == 7.0)
    res = np.stack([o.float().cpu().numpy() for o in outs]) if U else np.zeros((0, P), np.float32)
    return res, (None if n is None else n.cpu().numpy()[:U])


@pytest.mark.parametrize("in_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("W,P,U,norms", [
    (1, 1, 1, True), (2, 3, 2, False), (5, 1025, 1, True), (4, 4099, 3, False), (16, 70001, 5, True),
    (17, 33333, 2, True), (32, 50001, 4, False), (8, 300007, 1, True), (6, 20011, 70, True), (3, 9001, 200, False),
    # streams that need two launches although their tables are small enough for the kernel arguments
    (1, 5003, 32, True), (6, 5003, 30, True), (8, 5003, 29, True), (8, 5003, 32, True),
])
def test_reduce_random_shapes(in_dtype, out_dtype, W, P, U, norms):
    rng = np.random.default_rng(31 * W + U)
    rows = rand_rows(rng, W, P, in_dtype)
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    print(f"reduce W={W} P={P} U={U} norms={norms} in={in_dtype} out={out_dtype}", flush=True)
    eo, en = so.group_reduce(rows, offs, mem, wmode="stale", staleness=st, want_norms=True)
    out, n = run_reduce(rows, offs, mem, st, out_dtype, norms, P)
    tol = 4e-3 if "bf16" in (in_dtype, out_dtype) else 1e-6
    err = max(so.max_rel_err(out[u], eo[u]) for u in range(U))
    print(f"  err out={err:.3g}", flush=True)
    assert err <= tol
    if out_dtype == "bf16":      # each output is within half a bf16 ulp (plus fp32 noise) of the exact sum
        assert np.all(np.abs(out - eo) <= np.abs(eo) * 2.0 ** -8 * 1.001 + 1e-8)
    if norms:
        e_n = float(np.max(np.abs(n - en) / np.maximum(en, 1e-30)))
        assert e_n <= TOL[in_dtype]


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_reduce_unaligned_outputs_and_rows(out_dtype):
    rng = np.random.default_rng(5)
    W, P, U = 5, 12347, 3
    rows_big = rand_rows(rng, W, P + 1, "f32")
    offs, mem, st = rand_stream(rng, W, U, stale=2)
    rows = [r[1:] for r in rows_big]
    eo = so.group_reduce(rows, offs, mem, wmode="stale", staleness=st)
    drows = [r[1:] for r in to_dev_rows(rows_big)]          # 4 bytes off the 16-byte grid
    tdt = torch.float32 if out_dtype == "f32" else torch.bfloat16
    outs = [torch.zeros(P + 3, dtype=tdt, device="cuda")[3:] for _ in range(U)]
    star.star_group_reduce(outs, drows, star.UpdateStream(offs, mem, st), wmode="stale", **opts())
    torch.cuda.synchronize()
    tol = 4e-3 if out_dtype == "bf16" else 1e-6
    for u in range(U):
        assert so.max_rel_err(outs[u].float().cpu().numpy(), eo[u]) <= tol
    # aligned and unaligned runs agree bit for bit
    outs2 = [torch.zeros(P, dtype=tdt, device="cuda") for _ in range(U)]
    star.star_group_reduce(outs2, [r.clone() for r in drows], star.UpdateStream(offs, mem, st), wmode="stale", **opts())
    torch.cuda.synchronize()
    for a, b in zip(outs, outs2):
        assert torch.equal(a, b)


def test_reduce_parent_aggregation_feeds_update():
    """A parent adds its children's gradients to its own (plain sum, explicit
    coefficients 1), then the aggregate is used as one worker's report."""
    rng = np.random.default_rng(6)
    W, P = 4, 50021
    rows = rand_rows(rng, W, P, "f32")
    offs, mem = np.array([0, 3], np.int32), np.array([0, 2, 3], np.int32)
    cf = np.ones(3, np.float32)
    eo = so.group_reduce(rows, offs, mem, wmode="explicit", coeff=cf)
    out = [torch.zeros(P, device="cuda")]
    star.star_group_reduce(out, to_dev_rows(rows), star.UpdateStream(offs, mem, None, cf), wmode="explicit", **opts())
    torch.cuda.synchronize()
    assert so.max_rel_err(out[0].cpu().numpy(), eo[0]) <= 1e-6
    p0 = rng.standard_normal(P).astype(np.float32)
    p = torch.from_numpy(p0).cuda()
    v = torch.zeros(P, device="cuda")
    star.star_group_update(p, v, [out[0], to_dev_rows([rows[1]])[0]], star.UpdateStream([0, 2], [0, 1]),
                           lr=0.1, momentum_coef=0.9, **opts())
    torch.cuda.synchronize()
    ep, ev, _ = so.group_update(p0, np.zeros(P, np.float32), [eo[0].astype(np.float32), rows[1]], [0, 2], [0, 1],
                                lr=0.1, momentum_coef=0.9)
    assert so.max_rel_err(p.cpu().numpy(), ep) <= 1e-6


def test_reduce_empty_cases():
    e = torch.empty(0, device="cuda")
    n = torch.full((1,), 3.0, device="cuda")
    star.star_group_reduce([e], [e], star.UpdateStream([0, 1], [0]), norms_out=n, **opts())
    star.star_group_reduce([], [torch.ones(4, device="cuda")], star.UpdateStream([0], []), **opts())
    torch.cuda.synchronize()
    assert n.item() == 0.0
