"""Host-side logic of libstar, exercised without a GPU: the library loads, it
exports what include/star.h declares, argument checks return their status
codes before any device work, and the collapsed affine map agrees with the
step-by-step oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2512_09685_amd as star
from paper_2512_09685_amd import binding
from oracle import star_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "star.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(star_[a-z_]+)\s*\(", header))
    assert {"star_group_update", "star_group_norms", "star_group_reduce", "star_group_update_publish", "star_group_gram",
            "star_noise_scale", "star_select_mode_ps", "star_select_mode_ar", "star_plan_affine", "star_plan_choice", "star_plan_claims", "star_plan_even_split", "star_group_update_opt", "star_group_norms_opt",
            "star_group_reduce_opt", "star_group_gram_opt", "star_group_update_noalloc",
            "star_workspace_bytes", "star_last_error", "star_version", "star_shutdown"} <= names
    lib = star.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in star.star_version()


def _call_update(W=4, P=8, offsets=(0, 2), members=(0, 1), staleness=None, coeff=None, lr_arr=None, lr=0.1, mu=0.9,
                 wd=0.0, wmode=0, dtype=0, params=0x1000, momentum=0x2000, rows="fake", upd_null=False, hp_null=False):
    """Calls star_group_update with fake (never dereferenced) device addresses:
    every case here must be rejected before the device is touched."""
    lib = star.load_library()
    us = star.UpdateStream(offsets, members, staleness, coeff, lr_arr)
    hp = binding._HParams(lr, mu, wd, wmode, 0)
    ptrs = (ctypes.c_void_p * 32)(*([0x3000 + 0x100 * i for i in range(32)]))
    return lib.star_group_update(params, momentum, None if rows is None else ptrs, dtype, P, W,
                                 None if upd_null else ctypes.byref(us.c), None if hp_null else ctypes.byref(hp),
                                 None, None)


@pytest.mark.parametrize("kw,status", [
    (dict(upd_null=True), 1), (dict(hp_null=True), 1), (dict(rows=None), 1), (dict(params=None), 1),
    (dict(P=-1), 2), (dict(W=0), 2), (dict(W=33), 2),
    (dict(dtype=7), 5),
    (dict(offsets=(0, 0)), 3), (dict(offsets=(0, 2), members=(1, 1)), 3), (dict(members=(0, 4)), 3),
    (dict(members=(-1, 0)), 3), (dict(offsets=(1, 2)), 3), (dict(offsets=(0, 2, 1), members=(0, 1)), 3),
    (dict(lr=float("nan")), 4), (dict(mu=float("inf")), 4), (dict(wd=float("nan")), 4), (dict(wmode=9), 4),
    (dict(wmode=1, staleness=(0, -1)), 4), (dict(wmode=2, coeff=(1.0, float("inf"))), 4),
    (dict(wmode=2), 1), (dict(lr_arr=(float("nan"),)), 4),
])
def test_argument_checks(kw, status):
    assert _call_update(**kw) == status
    assert star.last_error() != ""


def test_empty_stream_and_empty_shard_are_no_ops():
    assert _call_update(offsets=(0,), members=()) == 0          # U = 0
    assert _call_update(P=0) == 0                                # P = 0, no norms
    assert star.last_error() == ""


def test_options_are_checked_before_anything_else():
    """star_options of the *_opt entry points: unknown kernel, unknown flag bits and a negative
    threshold are rejected (with fake device addresses: nothing may be touched)."""
    lib = star.load_library()
    us = star.UpdateStream((0, 2), (0, 1))
    hp = binding._HParams(0.1, 0.9, 0.0, 0, 0)
    ptrs = (ctypes.c_void_p * 32)(*([0x3000 + 0x100 * i for i in range(32)]))

    def call(kernel=0, flags=0, threshold=0, P=8):
        o = binding._Options(kernel, flags, threshold)
        return lib.star_group_update_opt(0x1000, 0x2000, ptrs, 0, P, 4, ctypes.byref(us.c), ctypes.byref(hp), None,
                                         None, 0, ctypes.byref(o), None)
    assert call(kernel=5) == 6 and "kernel" in star.last_error()
    assert call(kernel=-1) == 6
    assert call(flags=2) == 2 and "flags" in star.last_error()
    assert call(flags=-1) == 2
    assert call(flags=star.OPT_DIRECT_NORMS, P=0) == 0
    assert call(threshold=-1) == 2
    assert call(kernel=3, threshold=1, P=0) == 0            # valid options, empty shard: a no-op
    o = binding._Options(7, 0, 0)
    n = (ctypes.c_float * 1)()
    assert lib.star_group_norms_opt(ptrs, 0, 8, 4, ctypes.byref(us.c), 0, n, ctypes.byref(o), None) == 6
    assert lib.star_group_reduce_opt(ptrs, 0, ptrs, 0, 8, 4, ctypes.byref(us.c), 0, None, ctypes.byref(o), None) == 6
    assert lib.star_group_gram_opt(ptrs, 0, 8, 4, n, ctypes.byref(o), None) == 6
    info = binding._PlanInfo()
    assert lib.star_plan_choice(8, 4, 0, ctypes.byref(us.c), ctypes.byref(hp), 1, 0, ctypes.byref(o), ctypes.byref(info)) == 6


@pytest.mark.parametrize("claim", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 255, 256, 257, 512, 608, 1024])
def test_first_round_of_claims_tiles_the_front_of_the_shard(G, claim):
    """The fixed first claims are disjoint, leave no gap, start at tile 0 and end where the counter
    takes over; their sizes cycle 1, 2, .., claim (unequal, so that workgroups do not run in step)."""
    first, count, base = star.star_plan_claims(G, claim)
    assert count.tolist() == [1 + b % claim for b in range(G)]
    covered = np.zeros(base, np.int32)
    for b in range(G):
        covered[first[b]:first[b] + count[b]] += 1
    assert first[0] == 0 and (covered == 1).all() and int(count.sum()) == base


@pytest.mark.parametrize("G", [1, 2, 7, 256, 512, 1000])
def test_even_split_of_a_short_shard_covers_every_tile_once(G):
    """Short shards in queue order: workgroup b handles tiles [b n / G, (b+1) n / G).  The ranges follow one
    another without gap or overlap from tile 0 to tile n - 1 and their lengths differ by at most one, for
    fewer tiles than workgroups too (some then get none)."""
    for n in (0, 1, G - 1, G, G + 1, 3 * G + 5, 8 * G):
        if n < 0:
            continue
        first, count = star.star_plan_even_split(G, n)
        assert first[0] == 0 and int(first[-1]) + int(count[-1]) == n
        assert np.array_equal(first[1:], first[:-1] + count[:-1])
        assert count.min() >= 0 and count.max() - count.min() <= 1 and count.sum() == n
    lib = star.load_library()
    assert lib.star_plan_even_split(0, ctypes.c_int64(4), None, None) == 2
    assert lib.star_plan_even_split(4, ctypes.c_int64(-1), None, None) == 2
    assert lib.star_plan_even_split(4, ctypes.c_int64(4), None, None) == 1


def test_plan_claims_validation():
    lib = star.load_library()
    assert lib.star_plan_claims(0, 3, None, None, None) == 2
    assert lib.star_plan_claims(4, 0, None, None, None) == 2
    assert lib.star_plan_claims(4, 3, None, None, None) == 1


def _rand_stream(rng, W, U, stale=None):
    offs, mem = [0], []
    for _ in range(U):
        y = int(rng.integers(1, W + 1))
        mem += [int(x) for x in rng.permutation(W)[:y]]
        offs.append(len(mem))
    st = None if stale is None else rng.integers(0, stale + 1, size=len(mem)).astype(np.int32)
    return np.array(offs, np.int32), np.array(mem, np.int32), st


@pytest.mark.parametrize("seed,W,U,wd,scale", [(0, 5, 9, 0.0, False), (1, 16, 64, 1e-2, False), (2, 8, 33, 0.1, True),
                                               (3, 32, 128, 1e-4, False)])
def test_affine_map_equals_sequential_oracle(seed, W, U, wd, scale):
    rng = np.random.default_rng(seed)
    P = 50
    rows = [rng.standard_normal(P).astype(np.float32) for _ in range(W)]
    offs, mem, st = _rand_stream(rng, W, U, stale=4)
    lrs = rng.uniform(0.01, 0.2, U).astype(np.float32)
    p0 = rng.standard_normal(P).astype(np.float32)
    v0 = rng.standard_normal(P).astype(np.float32)
    us = star.UpdateStream(offs, mem, st, None, lrs)
    M, B = star.star_plan_affine(W, us, lr=0.0, momentum_coef=0.9, weight_decay=wd, wmode="stale",
                                 scale_lr_by_group=scale)
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.0, momentum_coef=0.9, weight_decay=wd, wmode="stale",
                              staleness=st, lr_per_update=lrs, scale_lr_by_group=scale, mode="f64")
    G = np.stack(rows).astype(np.float64)
    x0 = np.stack([p0, v0]).astype(np.float64)
    x = M @ x0 + B @ G
    np.testing.assert_allclose(x[0], p, rtol=0, atol=1e-12)
    np.testing.assert_allclose(x[1], v, rtol=0, atol=1e-12)


def test_affine_hand_case():
    # lr 0.5, mu 0.5, no decay, groups {0,1} then {1}:  p_2 = p_0 - 0.75*gbar_0 - 0.5*gbar_1 ... in worker terms
    us = star.UpdateStream([0, 2, 3], [0, 1, 1])
    M, B = star.star_plan_affine(2, us, lr=0.5, momentum_coef=0.5)
    # u0: v=gbar0, p=p-0.5 gbar0 ; u1: v=0.5 gbar0 + g1, p = p - 0.5 gbar0 - 0.25 gbar0 - 0.5 g1
    # gbar0 = (g0+g1)/2  ->  p: g0 coef -0.375, g1 coef -0.375-0.5 ; v: g0 0.25, g1 1.25
    np.testing.assert_allclose(M, [[1.0, -0.5 * 0.5 - 0.5 * 0.25], [0.0, 0.25]], atol=1e-15)
    np.testing.assert_allclose(B, [[-0.375, -0.875], [0.25, 1.25]], atol=1e-15)


def test_unused_rows_get_zero_coefficients():
    us = star.UpdateStream([0, 1, 3], [2, 0, 2])
    M, B = star.star_plan_affine(4, us, lr=0.1, momentum_coef=0.9)
    assert np.all(B[:, 1] == 0) and np.all(B[:, 3] == 0) and np.all(B[:, 0] != 0) and np.all(B[:, 2] != 0)


def test_plan_choice_one_update_is_literal_many_are_collapsed():
    one = star.UpdateStream([0, 4], [0, 1, 2, 3])
    c = star.star_plan_choice(1000, 4, "f32", one, lr=0.1, momentum_coef=0.9)
    assert (c["kernel"], c["fma_seq"], c["fma_affine"]) == (star.KERNEL_SEQ, 7.0, 12.0)
    assert c["launches"] == 1 and c["finishing_launches"] == 0 and c["tables_inline"] == 1 and c["queue_order"] == 0
    assert star.star_plan_choice(1000, 4, "bf16", one, lr=0.1, momentum_coef=0.9)["kernel"] == star.KERNEL_AFFINE
    rng = np.random.default_rng(0)
    offs, mem, _ = _rand_stream(rng, 16, 64)
    many = star.UpdateStream(offs, mem)
    c = star.star_plan_choice(100000, 16, "f32", many, lr=0.1, momentum_coef=0.9, want_norms=True)
    assert c["kernel"] == star.KERNEL_AFFINE_MFMA and c["fma_affine"] == 36 + 136 and c["fma_seq"] == len(mem) + 4 * 64
    assert c["queue_order"] == 1 and c["finishing_launches"] == 2      # the matrix-core kernel always takes the queue
    c = star.star_plan_choice(1000, 16, "f32", many, lr=0.1, momentum_coef=0.9, want_norms=True, kernel=star.KERNEL_AFFINE)
    assert c["kernel"] == star.KERNEL_AFFINE and c["queue_order"] == 0
    c = star.star_plan_choice(1000, 16, "f32", many, lr=0.1, momentum_coef=0.9, want_norms=True, kernel=star.KERNEL_SEQ)
    assert c["kernel"] == star.KERNEL_SEQ and c["launches"] == 3 and c["finishing_launches"] == 3 and c["tables_inline"] == 0
    # a shard of fewer than 4096 elements: norms from direct sums whatever the stream (a pass of its own beside the
    # collapsed update; the step-by-step kernel for the norms alone)
    c = star.star_plan_choice(1000, 16, "f32", many, lr=0.1, momentum_coef=0.9, want_norms=True)
    assert c["kernel"] == star.KERNEL_AFFINE and c["collapsed_update"] == 1 and c["launches"] == 1 + 3
    assert star.star_plan_choice(1000, 16, "f32", many, update=False, want_norms=True)["kernel"] == star.KERNEL_SEQ
    assert star.star_plan_choice(4096, 16, "f32", many, update=False, want_norms=True)["kernel"] == star.KERNEL_AFFINE_MFMA


def test_plan_choice_wide_fp32_rows_with_norms():
    """17 to 32 fp32 rows, update with norms: a short stream takes the collapsed update with direct norm sums
    (step-by-step kernel, one launch, queue order on long shards), a long one the Gram matrix on the matrix cores;
    bf16 rows, forced kernels and norms alone are not affected."""
    rng = np.random.default_rng(1)
    # 8 groups of 16 of the 32 workers: 8 * 17 = 136 multiply-adds for the direct norm sums, limit 4 * 32 + 48
    offs = np.arange(0, 129, 16, dtype=np.int32)
    mem = np.concatenate([np.sort(rng.choice(32, 16, replace=False)) for _ in range(8)]).astype(np.int32)
    short = star.UpdateStream(offs, mem)
    hp = dict(lr=0.1, momentum_coef=0.9, want_norms=True)
    c = star.star_plan_choice(50_000_000, 32, "f32", short, **hp)
    assert (c["kernel"], c["collapsed_update"], c["launches"], c["finishing_launches"], c["queue_order"]) == \
        (star.KERNEL_SEQ, 1, 1, 1, 1)
    assert c["fma_seq"] - 3 * 8 == 136
    # the same groups twice over: 272 multiply-adds, beyond the limit
    twice = star.UpdateStream(np.arange(0, 257, 16, dtype=np.int32), np.concatenate([mem, mem]))
    assert star.star_plan_choice(50_000_000, 32, "f32", twice, **hp)["kernel"] == star.KERNEL_AFFINE_MFMA
    # 20 rows: limit 128
    offs20 = np.arange(0, 81, 10, dtype=np.int32)
    mem20 = np.concatenate([np.sort(rng.choice(20, 10, replace=False)) for _ in range(8)]).astype(np.int32)
    assert star.star_plan_choice(1 << 20, 20, "f32", star.UpdateStream(offs20, mem20), **hp)["kernel"] == star.KERNEL_SEQ
    offs20 = np.arange(0, 8 * 16 + 1, 16, dtype=np.int32)
    mem20 = np.concatenate([np.sort(rng.choice(20, 16, replace=False)) for _ in range(8)]).astype(np.int32)
    assert star.star_plan_choice(1 << 20, 20, "f32", star.UpdateStream(offs20, mem20), **hp)["kernel"] == \
        star.KERNEL_AFFINE_MFMA
    assert star.star_plan_choice(50_000_000, 32, "bf16", short, **hp)["kernel"] == star.KERNEL_AFFINE_MFMA
    assert star.star_plan_choice(50_000_000, 32, "f32", short, kernel=star.KERNEL_AFFINE_MFMA, **hp)["kernel"] == \
        star.KERNEL_AFFINE_MFMA
    c = star.star_plan_choice(50_000_000, 32, "f32", short, kernel=star.KERNEL_SEQ, **hp)
    assert c["kernel"] == star.KERNEL_SEQ and c["collapsed_update"] == 0
    assert star.star_plan_choice(50_000_000, 32, "f32", short, update=False, want_norms=True)["kernel"] == \
        star.KERNEL_AFFINE_MFMA
    offs, mem, _ = _rand_stream(rng, 32, 64)
    c = star.star_plan_choice(50_000_000, 32, "f32", star.UpdateStream(offs, mem), **hp)
    assert c["kernel"] == star.KERNEL_AFFINE_MFMA and c["collapsed_update"] == 1
    offs, mem, _ = _rand_stream(rng, 16, 8)
    assert star.star_plan_choice(50_000_000, 16, "f32", star.UpdateStream(offs, mem), **hp)["kernel"] == \
        star.KERNEL_AFFINE_MFMA


def test_plan_choice_gram_route_for_few_rows():
    """Where the Gram matrix is formed when AUTO decides (measured crossovers, see gram_on_matrix_cores)."""
    def route(P, W, dt, update):
        us = star.UpdateStream(np.arange(0, 16 * W + 1, W, dtype=np.int32), np.tile(np.arange(W, dtype=np.int32), 16))
        c = star.star_plan_choice(P, W, dt, us, lr=0.1, momentum_coef=0.9, update=update, want_norms=True)
        return {star.KERNEL_AFFINE: "valu", star.KERNEL_AFFINE_MFMA: "mfma"}[c["kernel"]]   # (16 updates: not a stream for the literal kernel)
    Mi = 1 << 20
    # update with norms
    assert [route(4 * Mi, W, "f32", True) for W in (2, 6, 7, 8, 9, 16)] == ["valu"] * 4 + ["mfma"] * 2
    assert [route(64 * Mi, W, "f32", True) for W in (2, 6, 7, 8, 9)] == ["valu"] * 2 + ["mfma"] * 3
    assert [route(4 * Mi, W, "bf16", True) for W in (2, 3, 6, 8, 9)] == ["valu"] + ["mfma"] * 4
    assert [route(12 * Mi, W, "bf16", True) for W in (3, 4, 5, 6, 7, 8, 9)] == ["valu"] * 2 + ["mfma"] * 2 + ["valu"] * 2 + ["mfma"]
    assert [route(32 * Mi, W, "bf16", True) for W in (3, 4, 5, 6, 7, 8)] == ["valu"] + ["mfma"] * 5
    assert [route(64 * Mi, W, "bf16", True) for W in (3, 4, 6, 7, 8)] == ["valu"] * 3 + ["mfma"] * 2
    # norms alone
    assert [route(P, W, "f32", False) for P in (Mi, 96 * Mi) for W in (4, 8, 9, 16)] == ["valu", "valu", "mfma", "mfma"] * 2
    assert [route(12 * Mi, W, "bf16", False) for W in (2, 3, 4, 6, 7)] == ["valu"] + ["mfma"] * 4
    assert [route(32 * Mi, W, "bf16", False) for W in (2, 3, 4, 5, 6, 7)] == ["valu"] * 3 + ["mfma"] * 3
    assert [route(96 * Mi, W, "bf16", False) for W in (4, 5, 6, 7, 16)] == ["valu"] * 3 + ["mfma"] * 2


def test_plan_choice_short_streams_with_norms_take_the_literal_kernel():
    """Update with norms: up to 48 multiply-adds of stream (sum of y_u + 4) on a shard of up to 4 Mi elements (bf16
    rows: 16 Mi) the literal kernel (direct norms in the same pass, one finishing launch); with 17 to 32 fp32 rows up to 112
    multiply-adds at every length."""
    def choice(P, W, dt, U, norms=True):
        us = star.UpdateStream(np.arange(0, U * W + 1, W, dtype=np.int32), np.tile(np.arange(W, dtype=np.int32), U))
        return star.star_plan_choice(P, W, dt, us, lr=0.1, momentum_coef=0.9, want_norms=norms)
    Mi = 1 << 20
    for dt in ("f32", "bf16"):
        c = choice(Mi, 8, dt, 2)                       # 24 multiply-adds
        assert (c["kernel"], c["collapsed_update"], c["launches"], c["finishing_launches"]) == (star.KERNEL_SEQ, 0, 1, 1)
        assert choice(4 * Mi, 8, dt, 4)["kernel"] == star.KERNEL_SEQ          # 48
        assert choice(4 * Mi, 8, dt, 5)["kernel"] != star.KERNEL_SEQ          # 60
        assert choice((5 if dt == "f32" else 17) * Mi, 8, dt, 2)["kernel"] != star.KERNEL_SEQ    # too long a shard
    assert choice(16 * Mi, 8, "bf16", 2)["kernel"] == star.KERNEL_SEQ         # (bf16 rows: up to 16 Mi elements)
    assert choice(Mi, 32, "bf16", 1)["kernel"] == star.KERNEL_SEQ             # 36
    assert choice(Mi, 8, "bf16", 2, norms=False)["kernel"] == star.KERNEL_AFFINE
    # wide fp32 rows
    c = choice(64 * Mi, 32, "f32", 3)                  # 108: literal
    assert c["kernel"] == star.KERNEL_SEQ and c["collapsed_update"] == 0
    c = choice(64 * Mi, 32, "f32", 4)                  # 144: collapsed update with the norm walk (limit 4 * 32 + 48 on y_u + 1)
    assert c["kernel"] == star.KERNEL_SEQ and c["collapsed_update"] == 1
    assert choice(64 * Mi, 32, "bf16", 3)["kernel"] == star.KERNEL_AFFINE_MFMA


def test_plan_choice_direct_norms_option():
    """STAR_OPT_DIRECT_NORMS: the update stays collapsed and gets a direct norm pass beside it (one more
    launch over the rows and its finishing launch instead of the Gram matrix's two); norms alone go to the
    step-by-step kernel; a forced kernel and a call without norms ignore the flag."""
    us = star.UpdateStream(np.arange(0, 17, 2, dtype=np.int32), np.tile(np.arange(8, dtype=np.int32), 2))   # 8 groups of 2
    hp = dict(lr=0.1, momentum_coef=0.9)
    for dt in ("f32", "bf16"):
        gram = star.star_plan_choice(24 << 20, 8, dt, us, want_norms=True, **hp)
        direct = star.star_plan_choice(24 << 20, 8, dt, us, want_norms=True, direct_norms=True, **hp)
        assert gram["kernel"] in (star.KERNEL_AFFINE, star.KERNEL_AFFINE_MFMA) and gram["launches"] == 1
        assert gram["finishing_launches"] == 2
        assert direct["kernel"] == star.KERNEL_AFFINE and direct["collapsed_update"] == 1
        assert direct["launches"] == 2 and direct["finishing_launches"] == 1
        alone = star.star_plan_choice(24 << 20, 8, dt, us, update=False, want_norms=True, direct_norms=True, **hp)
        assert alone["kernel"] == star.KERNEL_SEQ
        forced = star.star_plan_choice(24 << 20, 8, dt, us, want_norms=True, direct_norms=True,
                                       kernel=star.KERNEL_AFFINE_MFMA, **hp)
        assert forced["kernel"] == star.KERNEL_AFFINE_MFMA and forced["launches"] == 1
        plain = star.star_plan_choice(24 << 20, 8, dt, us, direct_norms=True, **hp)
        assert plain == star.star_plan_choice(24 << 20, 8, dt, us, **hp)


def test_plan_choice_reports_the_kernels_of_the_five_workloads():
    """What bench.py labels its roofline with: the library's own answer, for every workload as it is timed."""
    import workloads
    expect = {"tiny": (star.KERNEL_AFFINE, 4, 0), "resnet50": (star.KERNEL_AFFINE, 8, 1),
              "bert_base": (star.KERNEL_AFFINE_MFMA, 16, 1), "vgg16": (star.KERNEL_AFFINE, 32, 1),
              "bert_large": (star.KERNEL_AFFINE_MFMA, 16, 1)}
    for name, (kernel, rows, queue) in expect.items():
        wl = workloads.WORKLOADS[name]
        s = workloads.make_update_stream(wl, 0, 0)
        us = star.UpdateStream(s["offsets"], s["members"], s["staleness"])
        c = star.star_plan_choice(wl.P, wl.W, wl.grad_dtype, us, lr=wl.lr, momentum_coef=wl.momentum,
                                  weight_decay=wl.weight_decay, wmode=wl.wmode, want_norms=wl.norms)
        assert (c["kernel"], c["rows_padded"], c["queue_order"]) == (kernel, rows, queue), (name, c)
        assert c["rows_used"] == wl.W and c["launches"] == 1 and c["grad_dtype"] == (0 if wl.grad_dtype == "f32" else 1)
        # a single update per call (every report applied on arrival): literal kernel on fp32 rows only
        one = star.UpdateStream(s["offsets"][:2], s["members"][:s["offsets"][1]],
                                None if s["staleness"] is None else s["staleness"][:s["offsets"][1]])
        c1 = star.star_plan_choice(wl.P, wl.W, wl.grad_dtype, one, lr=wl.lr, momentum_coef=wl.momentum,
                                   weight_decay=wl.weight_decay, wmode=wl.wmode, want_norms=False)
        assert c1["kernel"] == (star.KERNEL_SEQ if wl.grad_dtype == "f32" else star.KERNEL_AFFINE)
        # norms alone
        cn = star.star_plan_choice(wl.P, wl.W, wl.grad_dtype, us, wmode=wl.wmode, update=False, want_norms=True)
        valu = wl.W <= 8 if wl.grad_dtype == "f32" else wl.W <= 2      # (the five have 4, 8, 16 fp32 and 16, 32 bf16 rows)
        assert cn["kernel"] == (star.KERNEL_AFFINE if valu else star.KERNEL_AFFINE_MFMA)


def test_workspace_bytes_is_modest():
    assert star.star_workspace_bytes(0, 4, 4) == 0
    assert 0 < star.star_workspace_bytes(340_000_000, 16, 64) < 8 << 20


def test_group_reduce_argument_checks():
    lib = star.load_library()
    us = star.UpdateStream([0, 2], [0, 1])
    ptrs = (ctypes.c_void_p * 32)(*([0x3000 + 0x100 * i for i in range(32)]))
    outs = (ctypes.c_void_p * 1)(0x9000)
    call = lambda o, od, r, rd, P, W: lib.star_group_reduce(o, od, r, rd, P, W, ctypes.byref(us.c), 0, None, None)
    assert call(None, 0, ptrs, 0, 8, 4) == 1          # no outputs
    assert call(outs, 3, ptrs, 0, 8, 4) == 5          # output dtype
    assert call(outs, 0, ptrs, 9, 8, 4) == 5          # gradient dtype
    assert call(outs, 0, None, 0, 8, 4) == 1
    assert call(outs, 0, ptrs, 0, -2, 4) == 2
    assert call(outs, 0, ptrs, 0, 8, 1) == 3          # member id 1 outside [0, 1)
    assert call((ctypes.c_void_p * 1)(None), 0, ptrs, 0, 8, 4) == 1
    assert call(outs, 0, ptrs, 0, 0, 4) == 0          # empty shard: nothing to do


def test_noise_scale_host_function():
    g2, tr, phi = star.star_noise_scale(np.array([[9.0, 3.0], [3.0, 1.0]]), 8.0)      # rows (3) and (1)
    assert (g2, tr, phi) == (3.0, 16.0, 16.0 / 3.0)
    lib = star.load_library()
    lib.star_noise_scale.restype = ctypes.c_int
    g = (ctypes.c_double * 4)(9.0, 3.0, 3.0, 1.0)
    assert lib.star_noise_scale(ctypes.c_int32(1), g, ctypes.c_double(8.0), None, None, None) == 2
    assert lib.star_noise_scale(ctypes.c_int32(2), None, ctypes.c_double(8.0), None, None, None) == 1
    assert lib.star_noise_scale(ctypes.c_int32(2), g, ctypes.c_double(0.0), None, None, None) == 4
    lib.star_group_gram.restype = ctypes.c_int
    ptrs = (ctypes.c_void_p * 32)(*([0x3000 + 0x100 * i for i in range(32)]))
    assert lib.star_group_gram(ptrs, 0, ctypes.c_int64(8), ctypes.c_int32(33), ctypes.c_void_p(0x9000), None) == 2
    assert lib.star_group_gram(ptrs, 0, ctypes.c_int64(8), ctypes.c_int32(4), None, None) == 1


def test_affine_map_property_random_streams():
    """Property test: for arbitrary small streams and hyper-parameters the collapsed
    map reproduces the sequential oracle."""
    from hypothesis import given, settings, strategies as hst

    @settings(max_examples=60, deadline=None)
    @given(hst.integers(1, 8), hst.integers(1, 12), hst.integers(0, 2 ** 31 - 1), hst.floats(0.0, 0.99),
           hst.floats(0.0, 0.5), hst.booleans())
    def prop(W, U, seed, mu, wd, scale):
        rng = np.random.default_rng(seed)
        P = 7
        rows = [rng.standard_normal(P).astype(np.float32) for _ in range(W)]
        offs, mem, st = _rand_stream(rng, W, U, stale=3)
        lrs = rng.uniform(0.0, 0.3, U).astype(np.float32)
        p0, v0 = rng.standard_normal(P).astype(np.float32), rng.standard_normal(P).astype(np.float32)
        us = star.UpdateStream(offs, mem, st, None, lrs)
        M, B = star.star_plan_affine(W, us, lr=0.0, momentum_coef=mu, weight_decay=wd, wmode="stale",
                                     scale_lr_by_group=scale)
        p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.0, momentum_coef=mu, weight_decay=wd, wmode="stale",
                                  staleness=st, lr_per_update=lrs, scale_lr_by_group=scale, mode="f64")
        x = M @ np.stack([p0, v0]).astype(np.float64) + B @ np.stack(rows).astype(np.float64)
        np.testing.assert_allclose(x[0], p, rtol=0, atol=1e-11)
        np.testing.assert_allclose(x[1], v, rtol=0, atol=1e-11)

    prop()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_kernel_digest_ignores_comments_only():
    """bench.py keeps rocprofv3's measured HBM bytes together with a digest of the kernel sources and
    reports them only while the digest matches: it must move with the code and not with comments."""
    import importlib
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    bench = importlib.import_module("bench")
    real_open = open
    edits = {}

    def fake_open(path, mode="r", *a, **k):
        f = real_open(path, mode, *a, **k)
        if str(path).endswith("star_device.h") and "b" not in mode and edits:
            import io
            text = f.read()
            f.close()
            return io.StringIO(edits["fn"](text))
        return f

    base = bench.kernel_source_digest()
    import builtins
    try:
        builtins.open = fake_open
        edits["fn"] = lambda t: t.replace("namespace star {", "// a remark\nnamespace star {   /* another */", 1)
        assert bench.kernel_source_digest() == base
        edits["fn"] = lambda t: t.replace("constexpr int kGramFold = 64;", "constexpr int kGramFold = 32;", 1)
        assert bench.kernel_source_digest() != base
    finally:
        builtins.open = real_open


def test_header_is_plain_c_and_links(tmp_path):
    """include/star.h compiles as C (gcc -std=c99 -pedantic), a C program that takes the address of every
    declared entry point links against libstar.so, and its host-only calls run without a GPU."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "star.h")).read()
    names = sorted(set(re.findall(r"^(?:star_status|size_t|void|const char \*)\s*(star_[a-z_0-9]+)\s*\(", header, re.M)))
    assert "star_group_update" in names and "star_group_norms" in names and "star_version" in names
    src = tmp_path / "abi.c"
    body = "\n".join(f"    sink((void (*)(void))&{n});" for n in names)
    src.write_text(
        '#include "star.h"\n#include <stdio.h>\nstatic int count;\n'
        "static void sink(void (*f)(void)) { if (f) ++count; }\n"
        "int main(void) {\n" + body + "\n"
        "    { star_options o = {99, 0, 0}; star_plan_info info;\n"
        "      if (star_plan_choice(8, 2, STAR_F32, 0, 0, 1, 0, &o, &info) != STAR_ERR_KERNEL) return 2; }\n"
        "    { int64_t first[4]; int32_t cnt[4]; int64_t base;\n"
        "      if (star_plan_claims(4, 3, first, cnt, &base) != STAR_OK || base != 7) return 3; }\n"
        '    printf("%d %s\\n", count, star_version());\n    return 0;\n}\n')
    exe = tmp_path / "abi"
    lib_dir = os.path.dirname(star.library_path())
    star.load_library()          # builds the library if there is none
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src),
                        "-o", str(exe), "-L", lib_dir, "-lstar", "-Wl,-rpath," + lib_dir], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.split()[0] == str(len(names)), (r.returncode, r.stdout, r.stderr)


def test_host_planner_and_selector_under_sanitizers(tmp_path):
    """The pure-host sources (planner, mode selector) built with the address and undefined-behaviour
    sanitizers take random update streams, valid and broken, and random iteration times: every call
    returns a status and neither sanitizer reports anything (a report ends the program with an error)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2512_09685_amd", "csrc")
    exe = tmp_path / "host_fuzz"
    r = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                        "-I", os.path.join(root, "include"), "-I", csrc, os.path.join(root, "tests", "host_fuzz.cpp"),
                        os.path.join(csrc, "star_plan.cpp"), os.path.join(csrc, "star_select.cpp"), "-o", str(exe)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe), "20000", "10000"], capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout, r.stderr[-2000:])
    assert "plans accepted" in r.stdout and "selector calls accepted 20000" in r.stdout


def test_plan_choice_is_consistent_over_random_calls():
    """star_plan_choice over a few thousand random calls (streams, row counts, dtypes, shard lengths, norms,
    weightings with and without negative coefficients, options): whatever rule fires, the answer hangs together."""
    rng = np.random.default_rng(2024)
    seen = set()
    for _ in range(4000):
        W = int(rng.integers(1, 33))
        U = int(rng.choice([1, 2, 3, 4, 8, 16, 40, 200]))
        offs, mem, _ = _rand_stream(rng, W, U)
        explicit = rng.random() < 0.2
        cf = (rng.uniform(-1 if rng.random() < 0.5 else 0.01, 1, len(mem)).astype(np.float32)) if explicit else None
        us = star.UpdateStream(offs, mem, None, cf)
        P = int(rng.choice([1, 1000, 1 << 18, 1 << 20, 3 << 20, 5 << 20, 9 << 20, 17 << 20, 40 << 20, 70 << 20, 300 << 20]))
        dt = str(rng.choice(["f32", "bf16"]))
        update, norms = bool(rng.random() < 0.8), bool(rng.random() < 0.6)
        if not update:
            norms = True
        kw = dict(update=update, want_norms=norms, wmode="explicit" if explicit else "mean",
                  kernel=None if rng.random() < 0.7 else int(rng.integers(0, 4)),
                  queue_threshold=None if rng.random() < 0.8 else int(rng.choice([1, 1 << 40])),
                  direct_norms=bool(rng.random() < 0.15))
        c = star.star_plan_choice(P, W, dt, us, lr=0.1, momentum_coef=0.9, **kw)
        used = len(set(int(x) for x in mem))
        assert c["kernel"] in (star.KERNEL_SEQ, star.KERNEL_AFFINE, star.KERNEL_AFFINE_MFMA), (kw, c)
        assert c["rows_used"] == used and used <= c["rows_padded"] <= 32
        assert c["launches"] >= 1 and c["queue_order"] in (0, 1) and c["collapsed_update"] in (0, 1)
        assert (c["finishing_launches"] > 0) == norms, (kw, c)
        if c["kernel"] == star.KERNEL_AFFINE_MFMA:
            assert norms and c["queue_order"] == 1 and c["finishing_launches"] == 2
        if c["kernel"] == star.KERNEL_AFFINE:
            assert c["collapsed_update"] == (1 if update else 0)
            if norms and c["rows_padded"] > 16:      # no vector-register Gram beyond 16 rows: update plus a direct norm pass
                assert update and c["launches"] >= 2
        if c["kernel"] != star.KERNEL_SEQ and not update:
            assert c["launches"] == 1
        if not update:
            assert c["collapsed_update"] == 0
        if kw["kernel"] in (star.KERNEL_SEQ, star.KERNEL_AFFINE_MFMA) and (norms or kw["kernel"] == star.KERNEL_SEQ):
            assert c["kernel"] == kw["kernel"], (kw, c)
        if kw["queue_threshold"] == 1 << 40 and c["kernel"] != star.KERNEL_AFFINE_MFMA:
            assert c["queue_order"] == 0
        seen.add((c["kernel"], c["collapsed_update"], c["queue_order"], c["launches"] > 1))
    assert len(seen) >= 8       # the generator reaches the different routes
