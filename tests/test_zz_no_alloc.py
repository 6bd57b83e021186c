"""star_group_update_noalloc (the entry point whose workspace is a fixed array inside the library,
for callers that cannot allocate) against star_group_update, through the C ABI: same kernels, so the
state must come out bit for bit the same and the norms within the fp32 tolerance (they are equal in
practice).  Every case makes two calls in a row on the same GPU, the second with a smaller input, so
that the second call finds the first one's tables, partial sums and queue state in the array."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2512_09685_amd as star
from oracle import star_oracle as so

pytestmark = pytest.mark.gpu


def _stream(rng, W, U, stale=4):
    offs, mem = [0], []
    for _ in range(U):
        y = int(rng.integers(1, W + 1))
        mem += [int(x) for x in rng.permutation(W)[:y]]
        offs.append(len(mem))
    st = rng.integers(0, stale + 1, size=len(mem)).astype(np.int32)
    return np.array(offs, np.int32), np.array(mem, np.int32), st


def _rows(rng, W, P, dtype):
    rows = [torch.from_numpy((rng.standard_normal(P) * 1e-2).astype(np.float32)).cuda() for _ in range(W)]
    return [r.to(torch.bfloat16) for r in rows] if dtype == "bf16" else rows


def _both(W, P, U, dtype, norms, rng):
    """Runs the two entry points on the same inputs; returns what each left in (p, v, norms)."""
    rows = _rows(rng, W, P, dtype)
    offs, mem, st = _stream(rng, W, U)
    us = star.UpdateStream(offs, mem, st)
    p0 = torch.from_numpy((rng.standard_normal(P) * 0.02).astype(np.float32)).cuda()
    v0 = torch.from_numpy((rng.standard_normal(P) * 0.01).astype(np.float32)).cuda()
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="stale")
    out = []
    for fn in (star.star_group_update, star.star_group_update_noalloc):
        p, v = p0.clone(), v0.clone()
        n = torch.full((U,), -1.0, device="cuda") if norms else None
        torch.cuda.synchronize()
        fn(p, v, rows, us, norms_out=n, **hp)
        torch.cuda.synchronize()
        out.append((p, v, n))
    return out, (rows, offs, mem, st, p0, v0, hp)


# (first call, second and smaller call); both tile orders: the queue from 16 Mi elements on
CASES = [
    ((16, 300007, 24, "f32", True), (16, 70001, 7, "f32", True)),        # matrix-core Gram route
    ((4, 200003, 12, "f32", True), (3, 5001, 5, "f32", True)),           # vector-register Gram route
    ((32, 150001, 40, "bf16", True), (17, 33333, 9, "bf16", True)),      # wide tiles, bf16 rows
    ((8, 400003, 1, "f32", True), (8, 9001, 1, "f32", True)),            # a single update: step-by-step kernel
    ((12, 250001, 16, "bf16", False), (5, 1025, 3, "bf16", False)),      # no norms: nothing but the update
    ((8, 17 * 1024 * 1024 + 5, 6, "f32", True), (8, 16 * 1024 * 1024 + 1027, 6, "f32", False)),     # tiles from the queue
    ((32, 150001, 8, "f32", True), (20, 33333, 7, "f32", True)),         # wide fp32 rows: collapsed update, direct norms
    ((32, 150001, 3, "f32", True), (20, 33333, 2, "f32", True)),         # the same rows, very short streams: literal kernel
    ((32, 150001, 20, "f32", True), (20, 33333, 16, "f32", True)),       # the same rows, longer streams: matrix cores
]


@pytest.mark.parametrize("first,second", CASES)
def test_noalloc_matches_group_update_two_calls_in_a_row(first, second):
    rng = np.random.default_rng(99)
    for k, (W, P, U, dtype, norms) in enumerate((first, second)):
        print(f"noalloc call {k}: W={W} P={P} U={U} {dtype} norms={norms}", flush=True)
        (ref, got), (_, offs, mem, st, _, _, hp) = _both(W, P, U, dtype, norms, rng)
        if dtype == "f32" and W > 16 and norms:   # which of the two routes of wide fp32 rows the case exercises
            c = star.star_plan_choice(P, W, dtype, star.UpdateStream(offs, mem, st), want_norms=True, **hp)
            want = (star.KERNEL_SEQ, 0) if U <= 3 else ((star.KERNEL_SEQ, 1) if U <= 8 else (star.KERNEL_AFFINE_MFMA, 1))
            assert (c["kernel"], c["collapsed_update"]) == want
        assert torch.equal(ref[0], got[0]) and torch.equal(ref[1], got[1])
        if norms:
            a, b = ref[2].cpu().numpy(), got[2].cpu().numpy()
            assert np.all(a > 0) and np.max(np.abs(a - b) / a) <= 1e-6


def test_noalloc_signed_coefficients_two_passes():
    """Coefficients of both signs: the norms come from a direct pass beside the collapsed update, so the
    call uses the fixed array twice in a row (tables uploaded twice, queue cleared twice)."""
    rng = np.random.default_rng(11)
    W, P, U = 5, 17 * 1024 * 1024 + 77, 4
    rows = _rows(rng, W, P, "f32")
    offs, mem, _ = _stream(rng, W, U)
    cf = rng.uniform(-1, 1, len(mem)).astype(np.float32)
    us = star.UpdateStream(offs, mem, None, cf)
    p0 = torch.from_numpy((rng.standard_normal(P) * 0.02).astype(np.float32)).cuda()
    res = []
    for fn in (star.star_group_update, star.star_group_update_noalloc):
        p, v = p0.clone(), torch.zeros(P, device="cuda")
        n = torch.full((U,), -1.0, device="cuda")
        fn(p, v, rows, us, norms_out=n, lr=0.05, momentum_coef=0.9, weight_decay=1e-3, wmode="explicit")
        torch.cuda.synchronize()
        res.append((p, v, n))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    a, b = res[0][2].cpu().numpy(), res[1][2].cpu().numpy()
    assert np.all(a > 0) and np.max(np.abs(a - b) / a) <= 1e-6


def test_noalloc_against_the_oracle():
    rng = np.random.default_rng(7)
    W, P, U = 16, 123457, 20
    (ref, got), (rows, offs, mem, st, p0, v0, hp) = _both(W, P, U, "f32", True, rng)
    ep, ev, en = so.group_update(p0.cpu().numpy(), v0.cpu().numpy(), [r.cpu().numpy() for r in rows], offs, mem,
                                 staleness=st, want_norms=True, **hp)
    assert so.max_rel_err(got[0].cpu().numpy(), ep) <= 1e-6 and so.max_rel_err(got[1].cpu().numpy(), ev) <= 1e-6
    assert np.max(np.abs(got[2].cpu().numpy() - en) / en) <= 1e-6


def test_noalloc_rejects_streams_beyond_its_maximum():
    W, P, U = 2, 64, 257
    p = torch.ones(P, device="cuda")
    v = torch.zeros(P, device="cuda")
    rows = [torch.ones(P, device="cuda") for _ in range(W)]
    us = star.UpdateStream(np.arange(U + 1, dtype=np.int32), np.zeros(U, np.int32))
    with pytest.raises(star.StarError) as e:
        star.star_group_update_noalloc(p, v, rows, us, lr=0.1, momentum_coef=0.9)
    assert e.value.status == 2 and "256" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(p == 1) and torch.all(v == 0)          # nothing was enqueued
    us = star.UpdateStream(np.arange(257, dtype=np.int32), np.zeros(256, np.int32))
    star.star_group_update_noalloc(p, v, rows, us, lr=0.1, momentum_coef=0.9)      # 256 updates are accepted
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(p))


def test_noalloc_through_ctypes_directly():
    """The raw C call, no binding in between."""
    lib = star.load_library()
    P, W = 4099, 3
    rng = np.random.default_rng(3)
    rows = _rows(rng, W, P, "f32")
    p = torch.from_numpy(rng.standard_normal(P).astype(np.float32)).cuda()
    v = torch.zeros(P, device="cuda")
    p_ref, v_ref = p.clone(), v.clone()
    us = star.UpdateStream([0, 2, 3], [0, 2, 1])
    n = torch.zeros(2, device="cuda")
    n_ref = torch.zeros(2, device="cuda")
    star.star_group_update(p_ref, v_ref, rows, us, lr=0.1, momentum_coef=0.9, norms_out=n_ref)

    class HP(ctypes.Structure):
        _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                    ("wmode", ctypes.c_int32), ("scale", ctypes.c_int32)]
    hp = HP(0.1, 0.9, 0.0, 0, 0)
    ptrs = (ctypes.c_void_p * W)(*[r.data_ptr() for r in rows])
    rc = lib.star_group_update_noalloc(p.data_ptr(), v.data_ptr(), ptrs, 0, P, W, ctypes.byref(us.c), ctypes.byref(hp),
                                       n.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, star.last_error()
    torch.cuda.synchronize()
    assert torch.equal(p, p_ref) and torch.equal(v, v_ref) and torch.equal(n, n_ref)


def test_noalloc_under_graph_capture():
    """What the entry point is for: captured into a HIP graph (no allocation, no memset, no copy: kernels only)
    and replayed, with eager work and synchronisations between the replays; every replay must leave what the same
    number of eager calls leaves."""
    rng = np.random.default_rng(5)
    W, P, U = 16, 300007, 12
    rows = [torch.from_numpy((rng.standard_normal(P) * 1e-2).astype(np.float32)).cuda() for _ in range(W)]
    offs, mem = [0], []
    for _ in range(U):
        y = int(rng.integers(1, W + 1))
        mem += [int(x) for x in rng.permutation(W)[:y]]
        offs.append(len(mem))
    us = star.UpdateStream(offs, mem)
    hp = dict(lr=0.05, momentum_coef=0.9, weight_decay=1e-3)
    p0 = torch.from_numpy((rng.standard_normal(P) * 0.02).astype(np.float32)).cuda()
    # eager reference: the state after 1, 2, 3 calls (this also resolves the array's address outside the capture)
    p, v, n = p0.clone(), torch.zeros(P, device="cuda"), torch.zeros(U, device="cuda")
    ref = []
    for _ in range(3):
        star.star_group_update_noalloc(p, v, rows, us, norms_out=n, **hp)
        torch.cuda.synchronize()
        ref.append((p.clone(), v.clone(), n.clone()))
    # capture one call, replay three times from the same start
    p.copy_(p0)
    v.zero_()
    n.zero_()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        star.star_group_update_noalloc(p, v, rows, us, norms_out=n, **hp)
    torch.cuda.synchronize()
    assert torch.equal(p, p0)                     # capturing runs nothing
    scratch = torch.zeros(1 << 20, device="cuda")
    for k in range(3):
        g.replay()
        scratch.add_(1.0)                         # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(p, ref[k][0]) and torch.equal(v, ref[k][1]), f"replay {k}"
        assert torch.allclose(n, ref[k][2], rtol=1e-6, atol=0.0), f"replay {k}"
