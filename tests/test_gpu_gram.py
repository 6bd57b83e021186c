"""Gram matrix on the GPU against the oracle, and the noise-scale estimate
computed from it against the oracle's, which works straight from the rows."""
import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
from oracle import star_oracle as so
from gpu_util import opts, rand_rows, tile_order, to_dev_rows  # noqa: F401 (tile_order: autouse fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("mfma", [False, True])
@pytest.mark.parametrize("W,P", [(1, 5), (2, 1027), (5, 70001), (8, 300007), (16, 123457), (16, 3), (17, 40003),
                                 (23, 100001), (32, 70007), (32, 2)])
def test_gram_matrix(dtype, W, P, mfma):
    rng = np.random.default_rng(W * 7 + P)
    rows = rand_rows(rng, W, P, dtype)
    ref = so.gram(rows)
    out = torch.full((W, W), -1.0, dtype=torch.float64, device="cuda")
    kern = star.KERNEL_AFFINE_MFMA if mfma else star.KERNEL_AFFINE     # matrix cores / vector registers
    star.star_group_gram(to_dev_rows(rows), out, **opts(kern))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got, got.T)
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref)))          # |G_ab| <= sqrt(G_aa G_bb)
    err = float(np.max(np.abs(got - ref) / scale))
    print(f"gram W={W} P={P} {dtype}: err {err:.3g}", flush=True)
    assert err <= 1e-6


def test_gram_unaligned_rows_and_empty_shard():
    rng = np.random.default_rng(3)
    rows_big = rand_rows(rng, 4, 9002, "f32")
    d = [r[1:] for r in to_dev_rows(rows_big)]
    out = torch.zeros((4, 4), dtype=torch.float64, device="cuda")
    star.star_group_gram(d, out, **opts())
    torch.cuda.synchronize()
    ref = so.gram([r[1:] for r in rows_big])
    assert np.max(np.abs(out.cpu().numpy() - ref) / np.max(ref)) <= 1e-6
    e = torch.empty(0, device="cuda")
    out = torch.full((2, 2), 5.0, dtype=torch.float64, device="cuda")
    star.star_group_gram([e, e], out, **opts())
    torch.cuda.synchronize()
    assert torch.all(out == 0)


def test_noise_scale_from_device_gram():
    rng = np.random.default_rng(4)
    W, P, b, sigma = 16, 400003, 128.0, 0.4
    G = rng.standard_normal(P) * 0.02
    rows = [(G + rng.standard_normal(P) * sigma / np.sqrt(b)).astype(np.float32) for _ in range(W)]
    out = torch.zeros((W, W), dtype=torch.float64, device="cuda")
    star.star_group_gram(to_dev_rows(rows), out, **opts())
    torch.cuda.synchronize()
    g2, tr, phi = star.star_noise_scale(out.cpu().numpy(), b)
    eg2, etr, ephi = so.noise_scale(rows, b)
    # S - n2 and W n2 - S cancel leading digits of fp32-accumulated entries: 1e-4 is what survives
    assert abs(g2 / eg2 - 1) < 1e-4 and abs(tr / etr - 1) < 1e-4 and abs(phi / ephi - 1) < 2e-4
    assert abs(tr / (P * sigma ** 2) - 1) < 0.02          # and the estimate recovers the planted covariance
