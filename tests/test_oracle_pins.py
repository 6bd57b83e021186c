"""Pins for the CPU oracle: everything here fixes the oracle against something
other than itself -- hand-worked values, closed forms, the special cases the
paper defines (SSGD, ASGD), torch's SGD, exact rational arithmetic, invariants.
No GPU needed.
"""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import star_oracle as so

HERE = os.path.dirname(os.path.abspath(__file__))


def f32(x):
    return np.asarray(x, dtype=np.float32)


def rand_stream(rng, W, U, min_y=1, max_y=None, stale=None):
    max_y = max_y or W
    offs, mem = [0], []
    for _ in range(U):
        y = int(rng.integers(min_y, max_y + 1))
        mem += [int(x) for x in rng.permutation(W)[:y]]
        offs.append(len(mem))
    st = None if stale is None else rng.integers(0, stale + 1, size=len(mem)).astype(np.int32)
    return np.array(offs, np.int32), np.array(mem, np.int32), st


# ---------------------------------------------------------------- hand cases
with open(os.path.join(HERE, "golden", "hand_cases.json")) as fh:
    HAND = json.load(fh)["cases"]


@pytest.mark.parametrize("case", HAND, ids=[c["name"] for c in HAND])
@pytest.mark.parametrize("mode", ["exact", "f64", "f32step"])
def test_hand_cases(case, mode):
    if "rows_bf16_bits" in case:
        rows = [np.array(r, dtype=np.uint16) for r in case["rows_bf16_bits"]]
    else:
        rows = [f32(r) for r in case["rows"]]
    p, v, n = so.group_update(
        f32(case["params"]), f32(case["momentum"]), rows, case["offsets"], case["members"],
        lr=case["lr"], momentum_coef=case["mu"], weight_decay=case["wd"], wmode=case["wmode"],
        staleness=case.get("staleness"), coeff=case.get("coeff"), lr_per_update=case.get("lr_per_update"),
        scale_lr_by_group=case.get("scale_lr_by_group", False), want_norms=True, mode=mode)
    # every value is dyadic and small: all three modes must hit it exactly
    assert p.tolist() == case["expect_params"]
    assert v.tolist() == case["expect_momentum"]
    np.testing.assert_allclose(n, case["expect_norms"], rtol=1e-15)
    n2 = so.group_norms(rows, case["offsets"], case["members"], wmode=case["wmode"],
                        staleness=case.get("staleness"), coeff=case.get("coeff"))
    np.testing.assert_allclose(n2, case["expect_norms"], rtol=1e-15)


# ---------------------------------------------------------------- closed forms
def test_closed_form_no_momentum_no_decay():
    # mu = 0, wd = 0:  p_U = p_0 - sum_u lr_u * gbar_u
    rng = np.random.default_rng(1)
    W, P, U = 5, 37, 7
    rows = [f32(rng.standard_normal(P)) for _ in range(W)]
    offs, mem, _ = rand_stream(rng, W, U)
    lrs = f32(rng.uniform(0.01, 0.5, U))
    p0 = f32(rng.standard_normal(P))
    p, v, _ = so.group_update(p0, np.zeros(P, np.float32), rows, offs, mem, lr=1.0, momentum_coef=0.0,
                              lr_per_update=lrs, mode="f64")
    expect = p0.astype(np.float64)
    R = np.stack(rows).astype(np.float64)
    last = None
    for u in range(U):
        ids = mem[offs[u]:offs[u + 1]]
        last = R[ids].mean(axis=0)
        expect = expect - float(lrs[u]) * last
    np.testing.assert_allclose(p, expect, rtol=0, atol=1e-14)
    np.testing.assert_allclose(v, last, rtol=0, atol=1e-15)   # mu = 0: v is the last gbar


def test_closed_form_geometric_momentum():
    # wd = 0, constant lr, the same group every time:
    #   v_k = mu^k v_0 + gbar (1-mu^k)/(1-mu),   p_U = p_0 - lr sum_{k=1..U} v_k
    rng = np.random.default_rng(2)
    W, P, U, mu, lr = 3, 11, 9, 0.75, 0.125
    rows = [f32(rng.standard_normal(P)) for _ in range(W)]
    offs = np.arange(0, 2 * U + 1, 2, dtype=np.int32)
    mem = np.tile(np.array([2, 0], np.int32), U)
    p0, v0 = f32(rng.standard_normal(P)), f32(rng.standard_normal(P))
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=lr, momentum_coef=mu, mode="f64")
    gbar = (rows[0].astype(np.float64) + rows[2]) / 2
    p0, v0 = p0.astype(np.float64), v0.astype(np.float64)
    vk = [mu ** k * v0 + gbar * (1 - mu ** k) / (1 - mu) for k in range(1, U + 1)]
    np.testing.assert_allclose(v, vk[-1], rtol=0, atol=1e-13)
    np.testing.assert_allclose(p, p0 - lr * np.sum(vk, axis=0), rtol=0, atol=1e-13)


def test_closed_form_pure_decay():
    # all gradients zero, mu = 0:  p_U = p_0 (1 - lr wd)^U
    P, U, lr, wd = 6, 12, 0.5, 0.25
    rows = [np.zeros(P, np.float32) for _ in range(2)]
    offs = np.arange(U + 1, dtype=np.int32)
    mem = np.zeros(U, np.int32)
    p0 = f32([1, -2, 3, 0.5, 0, 8])
    p, v, n = so.group_update(p0, np.zeros(P, np.float32), rows, offs, mem, lr=lr, momentum_coef=0.0,
                              weight_decay=wd, want_norms=True, mode="f64")
    np.testing.assert_allclose(p, p0.astype(np.float64) * (1 - lr * wd) ** U, rtol=1e-14)
    assert np.all(n == 0)


def test_zero_lr_leaves_params():
    rng = np.random.default_rng(3)
    rows = [f32(rng.standard_normal(9)) for _ in range(3)]
    offs, mem, _ = rand_stream(rng, 3, 4)
    p0, v0 = f32(rng.standard_normal(9)), f32(rng.standard_normal(9))
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.0, momentum_coef=0.9, weight_decay=0.1)
    assert np.array_equal(p, p0)
    assert not np.array_equal(v, v0)


def test_norm_of_identical_rows():
    # every member holds the same row g:  ||gbar|| = ||g|| * sum of coefficients
    rng = np.random.default_rng(4)
    g = f32(rng.standard_normal(101))
    rows = [g.copy() for _ in range(4)]
    offs = np.array([0, 3, 4], np.int32)
    mem = np.array([3, 1, 0, 2], np.int32)
    st = np.array([0, 1, 3, 1], np.int32)
    n = so.group_norms(rows, offs, mem, wmode="stale", staleness=st)
    gn = np.linalg.norm(g.astype(np.float64))
    np.testing.assert_allclose(n, [gn * (1 + 0.5 + 0.25) / 3, gn * 0.5], rtol=1e-14)


# ---------------------------------------------------------------- SSGD / ASGD
def ssgd_step(p, v, rows, lr, mu, wd):
    """Synchronous SGD written on its own: add up every worker's gradient copy,
    divide by the number of workers, one momentum-SGD step."""
    total = np.zeros_like(p)
    for r in rows:
        total = total + r.astype(np.float64)
    g = total / len(rows)
    v = mu * v + (g + wd * p)
    return p - lr * v, v


def asgd_step(p, v, row, lr, mu, wd):
    """Asynchronous SGD written on its own: one worker's gradient, one step."""
    v = mu * v + (row.astype(np.float64) + wd * p)
    return p - lr * v, v


def test_full_group_is_ssgd():
    rng = np.random.default_rng(5)
    W, P, U = 6, 53, 5
    rows = [f32(rng.standard_normal(P)) for _ in range(W)]
    offs = np.arange(0, W * U + 1, W, dtype=np.int32)
    mem = np.concatenate([rng.permutation(W) for _ in range(U)]).astype(np.int32)
    p0, v0 = f32(rng.standard_normal(P)), f32(rng.standard_normal(P))
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.1, momentum_coef=0.9, weight_decay=1e-2, mode="f64")
    ep, ev = p0.astype(np.float64), v0.astype(np.float64)
    for _ in range(U):
        ep, ev = ssgd_step(ep, ev, rows, float(np.float32(0.1)), float(np.float32(0.9)), float(np.float32(1e-2)))
    np.testing.assert_allclose(p, ep, rtol=0, atol=1e-14)
    np.testing.assert_allclose(v, ev, rtol=0, atol=1e-14)


def test_singleton_group_is_asgd():
    rng = np.random.default_rng(6)
    W, P, U = 4, 29, 8
    rows = [f32(rng.standard_normal(P)) for _ in range(W)]
    who = rng.integers(0, W, U).astype(np.int32)
    offs = np.arange(U + 1, dtype=np.int32)
    p0, v0 = f32(rng.standard_normal(P)), np.zeros(P, np.float32)
    p, v, n = so.group_update(p0, v0, rows, offs, who, lr=0.05, momentum_coef=0.5, weight_decay=0.0,
                              want_norms=True, mode="f64")
    ep, ev = p0.astype(np.float64), v0.astype(np.float64)
    for u in range(U):
        ep, ev = asgd_step(ep, ev, rows[who[u]], float(np.float32(0.05)), 0.5, 0.0)
    np.testing.assert_allclose(p, ep, rtol=0, atol=1e-14)
    np.testing.assert_allclose(v, ev, rtol=0, atol=1e-14)
    np.testing.assert_allclose(n, [np.linalg.norm(rows[w].astype(np.float64)) for w in who], rtol=1e-14)


def test_stale_singleton_is_damped_asgd():
    rng = np.random.default_rng(7)
    P = 17
    rows = [f32(rng.standard_normal(P)) for _ in range(3)]
    p0 = f32(rng.standard_normal(P))
    p, v, _ = so.group_update(p0, np.zeros(P, np.float32), rows, [0, 1], [2], lr=0.25, momentum_coef=0.0,
                              wmode="stale", staleness=[3], mode="f64")
    np.testing.assert_allclose(p, p0 - 0.25 * rows[2].astype(np.float64) / 4, rtol=0, atol=1e-15)


# ---------------------------------------------------------------- torch.optim.SGD
@pytest.mark.parametrize("mu,wd", [(0.9, 1e-4), (0.0, 0.0), (0.5, 0.1)])
def test_against_torch_sgd(mu, wd):
    rng = np.random.default_rng(8)
    W, P, U = 7, 64, 12
    rows = [f32(rng.standard_normal(P) * 0.1) for _ in range(W)]
    offs, mem, _ = rand_stream(rng, W, U)
    lrs = f32(rng.uniform(0.01, 0.2, U))
    p0 = f32(rng.standard_normal(P))
    p, v, _ = so.group_update(p0, np.zeros(P, np.float32), rows, offs, mem, lr=1.0, momentum_coef=mu,
                              weight_decay=wd, lr_per_update=lrs, mode="f64")
    mu32, wd32 = float(np.float32(mu)), float(np.float32(wd))
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=1.0, momentum=mu32, weight_decay=wd32)
    R = torch.tensor(np.stack(rows), dtype=torch.float64)
    for u in range(U):
        ids = torch.tensor(mem[offs[u]:offs[u + 1]], dtype=torch.long)
        tp.grad = R[ids].mean(dim=0)
        opt.param_groups[0]["lr"] = float(lrs[u])
        opt.step()
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=0, atol=1e-13)
    if mu32 != 0.0:
        buf = opt.state[tp]["momentum_buffer"].numpy()
        np.testing.assert_allclose(v, buf, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- exact rational brute force
def affine_rational(p0, v0, rows, groups, coefs, lrs, mu, wd):
    """The U updates as one affine map, composed with exact fractions:
    state x=(p,v);  x' = A_u x + b_u gbar_u,  A_u=[[1-lr wd, -lr mu],[wd, mu]], b_u=(-lr, 1)."""
    out_p, out_v = [], []
    for j in range(len(p0)):
        M = [[Fraction(1), Fraction(0)], [Fraction(0), Fraction(1)]]
        c = [Fraction(0), Fraction(0)]
        for ids, cf, lr in zip(groups, coefs, lrs):
            gbar = sum((Fraction(k) * Fraction(float(rows[w][j])) for w, k in zip(ids, cf)), Fraction(0))
            A = [[1 - lr * wd, -lr * mu], [wd, mu]]
            b = [-lr * gbar, gbar]
            M = [[A[r][0] * M[0][k] + A[r][1] * M[1][k] for k in range(2)] for r in range(2)]
            c = [A[r][0] * c[0] + A[r][1] * c[1] + b[r] for r in range(2)]
        x = (Fraction(float(p0[j])), Fraction(float(v0[j])))
        out_p.append(M[0][0] * x[0] + M[0][1] * x[1] + c[0])
        out_v.append(M[1][0] * x[0] + M[1][1] * x[1] + c[1])
    return out_p, out_v


def test_exhaustive_tiny_cases_rational():
    # every ordered pair of non-empty groups over 3 workers, dyadic inputs:
    # fp64 evaluates these without rounding, so the oracle must equal the fraction
    rows = [f32([1.0, -0.5]), f32([0.25, 2.0]), f32([-3.0, 0.75])]
    p0, v0 = f32([1.0, -2.0]), f32([0.5, 0.0])
    mu, wd, lr = Fraction(1, 2), Fraction(1, 4), Fraction(1, 8)
    subsets = [list(s) for r in (1, 2, 3) for s in itertools.permutations(range(3), r)]
    # sizes 1, 2 use mean; size 3 would need 1/3 (not dyadic) -> use explicit dyadic coefficients there
    n = 0
    for g0, g1 in itertools.product(subsets, repeat=2):
        groups = [g0, g1]
        coefs = [[Fraction(1, 4) * (k + 1) for k in range(len(g))] for g in groups]
        mem = np.array(g0 + g1, np.int32)
        offs = np.array([0, len(g0), len(g0) + len(g1)], np.int32)
        cf = f32([float(c) for cc in coefs for c in cc])
        p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=float(lr), momentum_coef=float(mu),
                                  weight_decay=float(wd), wmode="explicit", coeff=cf, mode="f64")
        ep, ev = affine_rational(p0, v0, rows, groups, coefs, [lr, lr], mu, wd)
        assert [Fraction(float(x)) for x in p] == ep
        assert [Fraction(float(x)) for x in v] == ev
        n += 1
    assert n == 15 * 15


def test_mean_groups_rational_sizes_1_2_4():
    rng = np.random.default_rng(9)
    W, P = 4, 3
    rows = [f32(rng.integers(-8, 9, P) / 4.0) for _ in range(W)]
    p0, v0 = f32([1.0, -2.0, 0.5]), f32([0.5, 0.0, -1.0])
    groups = [[3, 1], [0, 1, 2, 3], [2], [1, 0]]
    coefs = [[Fraction(1, len(g))] * len(g) for g in groups]
    lrs = [Fraction(1, 4), Fraction(1, 8), Fraction(1, 2), Fraction(1, 4)]
    mem = np.array(sum(groups, []), np.int32)
    offs = np.cumsum([0] + [len(g) for g in groups]).astype(np.int32)
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.0, momentum_coef=0.5, weight_decay=0.125,
                              lr_per_update=f32([float(x) for x in lrs]), mode="f64")
    ep, ev = affine_rational(p0, v0, rows, groups, coefs, lrs, Fraction(1, 2), Fraction(1, 8))
    assert [Fraction(float(x)) for x in p] == ep
    assert [Fraction(float(x)) for x in v] == ev


# ---------------------------------------------------------------- invariants
def _setup(seed, W=6, P=40, U=6, stale=None):
    rng = np.random.default_rng(seed)
    rows = [f32(rng.standard_normal(P)) for _ in range(W)]
    offs, mem, st = rand_stream(rng, W, U, stale=stale)
    p0, v0 = f32(rng.standard_normal(P)), f32(rng.standard_normal(P))
    return rng, rows, offs, mem, st, p0, v0


def test_linear_in_gradients():
    rng, rows_a, offs, mem, st, p0, v0 = _setup(10, stale=3)
    rows_b = [f32(rng.standard_normal(40)) for _ in rows_a]
    kw = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.01, wmode="stale", staleness=st, mode="f64")
    z = [np.zeros(40, np.float32) for _ in rows_a]
    # use double-exact sums of the two gradient sets: a+b as float64 is not an fp32 row,
    # so test the affine property  x(a) + x(b) - x(0) = x(a+b)  with rows a, b chosen so a+b is exact in fp32
    rows_a = [f32(np.round(r * 64) / 64) for r in rows_a]
    rows_b = [f32(np.round(r * 64) / 64) for r in rows_b]
    rows_s = [a + b for a, b in zip(rows_a, rows_b)]
    pa, va, _ = so.group_update(p0, v0, rows_a, offs, mem, **kw)
    pb, vb, _ = so.group_update(p0, v0, rows_b, offs, mem, **kw)
    p0_, v0_, _ = so.group_update(p0, v0, z, offs, mem, **kw)
    ps, vs, _ = so.group_update(p0, v0, rows_s, offs, mem, **kw)
    np.testing.assert_allclose(pa + pb - p0_, ps, rtol=0, atol=1e-13)
    np.testing.assert_allclose(va + vb - v0_, vs, rtol=0, atol=1e-13)
    # homogeneity: scaling every gradient by 4 scales the response to the gradients by 4
    rows_4 = [4 * a for a in rows_a]
    p4, v4, n4 = so.group_update(p0, v0, rows_4, offs, mem, want_norms=True, **kw)
    _, _, n1 = so.group_update(p0, v0, rows_a, offs, mem, want_norms=True, **kw)
    np.testing.assert_allclose(p4 - p0_, 4 * (pa - p0_), rtol=0, atol=1e-13)
    np.testing.assert_allclose(n4, 4 * n1, rtol=1e-14)


def test_member_order_does_not_matter():
    rng, rows, offs, mem, st, p0, v0 = _setup(11, stale=4)
    kw = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.01, wmode="stale", want_norms=True, mode="f64")
    p, v, n = so.group_update(p0, v0, rows, offs, mem, staleness=st, **kw)
    mem2, st2 = mem.copy(), st.copy()
    for u in range(len(offs) - 1):
        perm = rng.permutation(offs[u + 1] - offs[u]) + offs[u]
        mem2[offs[u]:offs[u + 1]] = mem[perm]
        st2[offs[u]:offs[u + 1]] = st[perm]
    p2, v2, n2 = so.group_update(p0, v0, rows, offs, mem2, staleness=st2, **kw)
    np.testing.assert_allclose(p2, p, rtol=0, atol=1e-14)
    np.testing.assert_allclose(v2, v, rtol=0, atol=1e-14)
    np.testing.assert_allclose(n2, n, rtol=1e-14)


def test_worker_relabelling():
    rng, rows, offs, mem, st, p0, v0 = _setup(12)
    perm = rng.permutation(len(rows))            # new id of old worker w is perm[w]
    rows2 = [None] * len(rows)
    for w, r in enumerate(rows):
        rows2[perm[w]] = r
    kw = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.01, mode="f64")
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, **kw)
    p2, v2, _ = so.group_update(p0, v0, rows2, offs, perm[mem].astype(np.int32), **kw)
    assert np.array_equal(p, p2) and np.array_equal(v, v2)


def test_batch_split_carries_state():
    rng, rows, offs, mem, st, p0, v0 = _setup(13, U=9, stale=2)
    kw = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.01, wmode="stale")
    k = 4
    for mode, exact in (("f64", True), ("f32step", True), ("exact", False)):
        p, v, n = so.group_update(p0, v0, rows, offs, mem, staleness=st, want_norms=True, mode=mode, **kw)
        pa, va, na = so.group_update(p0, v0, rows, offs[:k + 1], mem[:offs[k]], staleness=st[:offs[k]],
                                     want_norms=True, mode=mode, **kw)
        pb, vb, nb = so.group_update(pa, va, rows, offs[k:] - offs[k], mem[offs[k]:], staleness=st[offs[k]:],
                                     want_norms=True, mode=mode, **kw)
        if exact:
            assert np.array_equal(p, pb) and np.array_equal(v, vb)
        else:   # one extra fp32 rounding at the split
            np.testing.assert_allclose(pb, p, rtol=3e-7, atol=1e-7)
            np.testing.assert_allclose(vb, v, rtol=3e-7, atol=1e-7)
        np.testing.assert_allclose(np.concatenate([na, nb]), n, rtol=1e-15)


def test_norms_match_numpy_and_standalone():
    rng, rows, offs, mem, st, p0, v0 = _setup(14, P=257, stale=5)
    _, _, n = so.group_update(p0, v0, rows, offs, mem, lr=0.1, momentum_coef=0.9, weight_decay=0.3,
                              wmode="stale", staleness=st, want_norms=True)
    n2 = so.group_norms(rows, offs, mem, wmode="stale", staleness=st)
    assert np.array_equal(n, n2)            # weight decay must not enter the norm
    R = np.stack(rows).astype(np.float64)
    for u in range(len(offs) - 1):
        ids = mem[offs[u]:offs[u + 1]]
        a = 1.0 / (1.0 + st[offs[u]:offs[u + 1]])
        gbar = (a[:, None] * R[ids]).sum(axis=0) / len(ids)
        np.testing.assert_allclose(n[u], np.linalg.norm(gbar), rtol=1e-13)


def test_lr_scaling_rule():
    rng, rows, offs, mem, st, p0, v0 = _setup(15, W=8, U=7)
    W = len(rows)
    kw = dict(momentum_coef=0.9, weight_decay=0.01, mode="f64")
    y = np.diff(offs).astype(np.float64)
    base = float(np.float32(0.25))
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.25, scale_lr_by_group=True, **kw)
    # the same as handing in lr*y/N per update (values chosen exactly representable: N = 8)
    p2, v2, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.0, lr_per_update=f32(base * y / W), **kw)
    assert np.array_equal(p, p2) and np.array_equal(v, v2)
    # y = N leaves the rate alone
    offs_full = np.array([0, W], np.int32)
    memf = np.arange(W, dtype=np.int32)
    a = so.group_update(p0, v0, rows, offs_full, memf, lr=0.25, scale_lr_by_group=True, **kw)
    b = so.group_update(p0, v0, rows, offs_full, memf, lr=0.25, scale_lr_by_group=False, **kw)
    assert np.array_equal(a[0], b[0])


def test_bf16_rows_equal_their_float_values():
    rng = np.random.default_rng(16)
    W, P = 5, 33
    bits = [rng.integers(0, 1 << 16, P).astype(np.uint16) for _ in range(W)]
    for b in bits:                       # avoid inf/nan exponents
        b[(b & 0x7F80) == 0x7F80] = 0x3F80
    as_f32 = [(b.astype(np.uint32) << 16).view(np.float32) for b in bits]
    small = [np.where(np.abs(a) < 1e3, a, np.float32(1.0)) for a in as_f32]
    bits = [(a.view(np.uint32) >> 16).astype(np.uint16) for a in small]
    offs, mem, _ = rand_stream(rng, W, 5)
    p0, v0 = f32(rng.standard_normal(P)), np.zeros(P, np.float32)
    kw = dict(lr=0.01, momentum_coef=0.9, weight_decay=0.0, want_norms=True, mode="f64")
    a = so.group_update(p0, v0, bits, offs, mem, **kw)
    b = so.group_update(p0, v0, small, offs, mem, **kw)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_stepwise_fp32_close_to_exact():
    import workloads
    wl = workloads.WORKLOADS["tiny"].scaled(4099)
    rows = workloads.rows_to_numpy(workloads.make_grad_rows(wl, 0))
    p0 = workloads.make_params(wl, 0).numpy()
    st = workloads.make_update_stream(wl, 0)
    kw = dict(lr=wl.lr, momentum_coef=wl.momentum, weight_decay=wl.weight_decay)
    pe, ve, _ = so.group_update(p0, np.zeros_like(p0), rows, st["offsets"], st["members"], mode="exact", **kw)
    ps, vs, _ = so.group_update(p0, np.zeros_like(p0), rows, st["offsets"], st["members"], mode="f32step", **kw)
    assert so.max_rel_err(ps, pe) < 1e-6
    assert so.max_rel_err(vs, ve) < 1e-6
    assert not np.array_equal(ps, pe) or not np.array_equal(vs, ve)   # they are different computations


def test_exact_mode_rounds_once():
    rng, rows, offs, mem, st, p0, v0 = _setup(17, U=20)
    kw = dict(lr=0.1, momentum_coef=0.9, weight_decay=0.01)
    p64, v64, _ = so.group_update(p0, v0, rows, offs, mem, mode="f64", **kw)
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, mode="exact", **kw)
    assert np.array_equal(p, p64.astype(np.float32)) and np.array_equal(v, v64.astype(np.float32))


@pytest.mark.parametrize("offs,mem", [([0, 2], [1, 1]), ([0, 0], []), ([0, 1], [5]), ([0, 1], [-1])])
def test_malformed_groups_rejected(offs, mem):
    rows = [np.zeros(3, np.float32) for _ in range(3)]
    with pytest.raises(ValueError):
        so.group_update(np.zeros(3, np.float32), np.zeros(3, np.float32), rows, offs, mem, lr=0.1,
                        momentum_coef=0.9)


def test_empty_stream_and_empty_shard():
    rows = [np.ones(3, np.float32)]
    p0 = f32([1, 2, 3])
    p, v, n = so.group_update(p0, p0, rows, [0], [], lr=0.1, momentum_coef=0.9, want_norms=True)
    assert np.array_equal(p, p0) and np.array_equal(v, p0) and n.size == 0
    e = np.zeros(0, np.float32)
    p, v, n = so.group_update(e, e, [e], [0, 1], [0], lr=0.1, momentum_coef=0.9, want_norms=True)
    assert p.size == 0 and n.tolist() == [0.0]


# ---------------------------------------------------------------- aggregation without the optimizer step
def test_reduce_hand_values():
    # rows 0.5 and -0.25: group {0,1} mean 0.125; group {1} -> -0.25; stale weight 1/(1+1) on it -> -0.125
    rows = [f32([0.5, 1.0]), f32([-0.25, 3.0])]
    out, n = so.group_reduce(rows, [0, 2, 3], [0, 1, 1], want_norms=True)
    assert out.tolist() == [[0.125, 2.0], [-0.25, 3.0]]
    np.testing.assert_allclose(n, [np.hypot(0.125, 2.0), np.hypot(0.25, 3.0)], rtol=1e-15)
    out = so.group_reduce(rows, [0, 2, 3], [0, 1, 1], wmode="stale", staleness=[0, 0, 1])
    assert out[1].tolist() == [-0.125, 1.5]
    out = so.group_reduce(rows, [0, 2], [1, 0], wmode="explicit", coeff=[2.0, 0.5])   # listed order: row 1 gets 2.0
    assert out[0].tolist() == [-0.25, 6.5]


def test_reduce_matches_numpy_and_norms_entry():
    rng, rows, offs, mem, st, p0, v0 = _setup(21, W=7, P=61, U=9, stale=4)
    out, n = so.group_reduce(rows, offs, mem, wmode="stale", staleness=st, want_norms=True)
    R = np.stack(rows).astype(np.float64)
    for u in range(len(offs) - 1):
        ids = mem[offs[u]:offs[u + 1]]
        a = 1.0 / (1.0 + st[offs[u]:offs[u + 1]])
        np.testing.assert_allclose(out[u], (a[:, None] * R[ids]).sum(axis=0) / len(ids), rtol=0, atol=1e-15)
        np.testing.assert_allclose(n[u], np.linalg.norm(out[u]), rtol=1e-14)
    assert np.array_equal(n, so.group_norms(rows, offs, mem, wmode="stale", staleness=st))


def test_reduce_feeds_a_plain_sgd_step():
    # mu = 0, wd = 0: one update is p - lr * (aggregated gradient)
    rng, rows, offs, mem, st, p0, v0 = _setup(22, U=1)
    out = so.group_reduce(rows, offs, mem)
    p, v, _ = so.group_update(p0, v0, rows, offs, mem, lr=0.25, momentum_coef=0.0, mode="f64")
    np.testing.assert_allclose(p, p0.astype(np.float64) - 0.25 * out[0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(v, out[0], rtol=0, atol=1e-15)


def test_reduce_bf16_rows_and_full_group_mean():
    bits = [np.array([0x3F00, 0x4000], np.uint16), np.array([0xBE80, 0x3F80], np.uint16)]   # 0.5, 2 | -0.25, 1
    out = so.group_reduce(bits, [0, 2], [0, 1])
    assert out[0].tolist() == [0.125, 1.5]


# ---------------------------------------------------------------- Gram matrix and noise scale
def test_gram_matches_matrix_product_and_norm_identity():
    rng, rows, offs, mem, st, p0, v0 = _setup(23, W=6, P=301, U=5, stale=3)
    G = so.gram(rows)
    R = np.stack(rows).astype(np.float64)
    np.testing.assert_allclose(G, R @ R.T, rtol=1e-13)
    assert np.array_equal(G, G.T)
    # || sum_w c_w g_w ||^2 = c^T Gamma c for every group of a stream
    n = so.group_norms(rows, offs, mem, wmode="stale", staleness=st)
    for u in range(len(offs) - 1):
        c = np.zeros(6)
        ids = mem[offs[u]:offs[u + 1]]
        c[ids] = 1.0 / (1.0 + st[offs[u]:offs[u + 1]]) / len(ids)
        np.testing.assert_allclose(n[u] ** 2, c @ G @ c, rtol=1e-12)
    bits = [np.array([0x3F00, 0x4000], np.uint16), np.array([0xBE80, 0x3F80], np.uint16)]   # (0.5, 2), (-0.25, 1)
    assert so.gram(bits).tolist() == [[4.25, 1.875], [1.875, 1.0625]]


def test_noise_scale_hand_case_and_recovery():
    # two workers, one element: g = 3 and 1: S = 5, |gbar|^2 = 4 -> tr = b*(5-4)*2 = 2b, |G|^2 = 2*4 - 5 = 3
    g2, tr, phi = so.noise_scale([f32([3.0]), f32([1.0])], 8.0)
    assert (g2, tr, phi) == (3.0, 16.0, 16.0 / 3.0)
    # synthetic gradients with known mean and per-sample covariance sigma^2 I
    rng = np.random.default_rng(0)
    W, P, b, sigma = 16, 20000, 32.0, 0.5
    G = rng.standard_normal(P) * 0.05
    rows = [(G + rng.standard_normal(P) * sigma / np.sqrt(b)).astype(np.float32) for _ in range(W)]
    g2, tr, phi = so.noise_scale(rows, b)
    assert abs(tr / (P * sigma ** 2) - 1) < 0.03 and abs(g2 / float(G @ G) - 1) < 0.1
