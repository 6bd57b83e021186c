"""Fused parameter publish: the copy written in the update pass equals the
updated parameters (fp32: same bits; bf16: round to nearest even of them), and
the update itself is unchanged."""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
from oracle import star_oracle as so
from gpu_util import TOL, opts, rand_rows, rand_stream, tile_order, to_dev_rows  # noqa: F401 (tile_order: autouse fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("pub", ["f32", "bf16"])
@pytest.mark.parametrize("kern", [star.KERNEL_SEQ, star.KERNEL_AFFINE, None])
@pytest.mark.parametrize("W,P,U,dtype,norms,shift", [
    (4, 5, 3, "f32", False, 0), (8, 70001, 12, "f32", True, 0), (16, 123457, 20, "bf16", True, 0),
    (32, 40003, 6, "bf16", True, 0), (3, 9001, 300, "f32", True, 0), (5, 30011, 7, "f32", False, 1),
    (24, 30011, 5, "f32", True, 0),      # the library's own choice here: collapsed update with direct norm sums
])
def test_publish(pub, kern, W, P, U, dtype, norms, shift):
    rng = np.random.default_rng(17 * W + U)
    rows = rand_rows(rng, W, P, dtype, std=1e-3 if U > 100 else 1e-2)
    offs, mem, st = rand_stream(rng, W, U, stale=3)
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    v0 = (rng.standard_normal(P) * 0.01).astype(np.float32)
    hp = dict(lr=0.01, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    us = star.UpdateStream(offs, mem, st)
    # reference run without publish
    p_ref, v_ref = torch.from_numpy(p0).cuda(), torch.from_numpy(v0).cuda()
    n_ref = torch.zeros(U, device="cuda") if norms else None
    drows = to_dev_rows(rows)
    star.star_group_update(p_ref, v_ref, drows, us, norms_out=n_ref, **opts(kern), **hp)
    # run with publish (optionally off the 16-byte grid)
    p, v = torch.from_numpy(p0).cuda(), torch.from_numpy(v0).cuda()
    n = torch.zeros(U, device="cuda") if norms else None
    tdt = torch.float32 if pub == "f32" else torch.bfloat16
    backing = torch.full((P + 8,), 3.0, dtype=tdt, device="cuda")
    out = backing[shift:shift + P]
    star.star_group_update_publish(p, v, drows, us, out, norms_out=n, **opts(kern), **hp)
    torch.cuda.synchronize()
    assert torch.equal(p, p_ref) and torch.equal(v, v_ref)
    if norms:
        assert torch.equal(n, n_ref)
    assert torch.all(backing[:shift] == 3.0) and torch.all(backing[shift + P:] == 3.0)
    if pub == "f32":
        assert torch.equal(out, p)
    else:
        assert torch.equal(out.cpu(), p.cpu().to(torch.bfloat16))      # torch's CPU conversion rounds to nearest even
    ep, ev, _ = so.group_update(p0, v0, rows, offs, mem, staleness=st, **hp)
    tol = 4e-3 if "bf16" in (pub, dtype) else 1e-6
    assert so.max_rel_err(out.float().cpu().numpy(), ep) <= tol


def test_publish_special_values_round_to_nearest_even():
    """bf16 publish of chosen finite bit patterns: ties to even both ways, just
    below / above a tie, overflow to infinity, a denormal, -0, carries into the exponent."""
    vals = np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F7FFFFF,
                     0x00000001, 0x80000000, 0x3FFFFFFF, 0x477FE000], dtype=np.uint32)
    expect = np.array([0x3F80, 0x3F82, 0x3F80, 0x3F81, 0x7F80,
                       0x0000, 0x8000, 0x4000, 0x4780], dtype=np.uint16)
    P = vals.size
    p = torch.from_numpy(vals.view(np.float32).copy()).cuda()
    v = torch.zeros(P, device="cuda")
    rows = [torch.zeros(P, device="cuda")]
    out = torch.zeros(P, dtype=torch.bfloat16, device="cuda")
    # lr = 0: the update leaves params alone, publish converts them
    star.star_group_update_publish(p, v, rows, star.UpdateStream([0, 1], [0]), out, lr=0.0, momentum_coef=0.0, **opts())
    torch.cuda.synchronize()
    got = out.cpu().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, expect)
