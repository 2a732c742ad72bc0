"""Pins for the oracle's momentum-SGD step and elastic-averaging step (Section 4:
momentum SGD as the optimiser; EASGD with moving rate alpha)."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from exact_arith import exact_round_f32 as rn, fr


# ---------------------------------------------------------------- momentum SGD

def test_plain_descent_when_momentum_and_decay_are_zero(oracle_mod):
    rng = np.random.default_rng(1)
    n, lr = 10_000, 0.01
    w0 = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = (rng.standard_normal(n) * 0.01).astype(np.float32)
    w, v = w0.copy(), (rng.standard_normal(n)).astype(np.float32)   # v must not matter
    oracle_mod.sgd_momentum(g, w, v, lr, 0.0, 0.0)
    ref = w0.astype(np.float64) - lr * g.astype(np.float64)
    assert np.max(np.abs(w - ref)) <= 2.0 ** -24 * np.max(np.abs(ref)) * 2
    assert np.allclose(v, -np.float32(lr) * g, rtol=1e-7, atol=0)


def test_constant_gradient_closed_form(oracle_mod):
    """wd = 0, constant g: v_t = -lr g (1 - mu^t)/(1 - mu), w_t = w_0 + sum v."""
    n, lr, mu, T = 1000, 0.01, 0.9, 25
    rng = np.random.default_rng(2)
    g = (rng.standard_normal(n) * 0.01).astype(np.float32)
    w0 = (rng.standard_normal(n) * 0.05).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, np.float32)
    g64 = g.astype(np.float64)
    lr64, mu64 = float(np.float32(lr)), float(np.float32(mu))
    for t in range(1, T + 1):
        oracle_mod.sgd_momentum(g, w, v, lr, mu, 0.0)
        v_ref = -lr64 * g64 * (1 - mu64 ** t) / (1 - mu64)
        assert np.max(np.abs(v - v_ref)) <= 1e-6 * np.max(np.abs(v_ref))
    geo = (T - mu64 * (1 - mu64 ** T) / (1 - mu64)) / (1 - mu64)
    w_ref = w0.astype(np.float64) - lr64 * g64 * geo
    assert np.max(np.abs(w - w_ref)) <= 1e-6 * np.max(np.abs(w_ref))


@pytest.mark.parametrize("wd", [0.0, 5e-4])
def test_against_torch_optim_sgd_on_cpu(oracle_mod, wd):
    """Library special case.  torch keeps a buffer b <- mu b + (g + wd w) and
    steps w <- w - lr b; with constant lr that is v = -lr b."""
    n, lr, mu, T = 20_000, 0.01, 0.9, 10
    rng = np.random.default_rng(3)
    w0 = (rng.standard_normal(n) * 0.05).astype(np.float32)
    w, v = w0.copy(), np.zeros(n, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd, dampening=0,
                          nesterov=False)
    for t in range(T):
        g = (rng.standard_normal(n) * 0.01).astype(np.float32)
        oracle_mod.sgd_momentum(g, w, v, lr, mu, wd)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        tw = p.detach().numpy()
        err = np.abs(w - tw)
        assert np.all((err <= 1e-6 * np.abs(tw)) | (err <= 1e-7)), t
    buf = opt.state[p]["momentum_buffer"].numpy()
    assert np.allclose(v, -np.float32(lr) * buf, rtol=1e-5, atol=1e-9)
    assert np.max(np.abs(w - w0)) > 1e-4


def test_bounded_by_double_precision_recurrence(oracle_mod):
    n, lr, mu, wd, T = 5000, 0.01, 0.9, 5e-4, 10
    rng = np.random.default_rng(4)
    w = (rng.standard_normal(n) * 0.01).astype(np.float32)
    v = np.zeros(n, np.float32)
    w64, v64 = w.astype(np.float64), v.astype(np.float64)
    lr64, mu64, wd64 = (float(np.float32(t)) for t in (lr, mu, wd))
    for _ in range(T):
        g = (rng.standard_normal(n) * 0.01).astype(np.float32)
        oracle_mod.sgd_momentum(g, w, v, lr, mu, wd)
        v64 = mu64 * v64 - lr64 * (g.astype(np.float64) + wd64 * w64)
        w64 = w64 + v64
    err = np.abs(w - w64)
    assert np.all((err <= 1e-6 * np.abs(w64)) | (err <= 1e-7))


def test_half_gradient_is_widened_exactly(oracle_mod):
    rng = np.random.default_rng(5)
    n = 10_000
    a16 = (rng.standard_normal(n) * 0.01).astype(np.float16)
    w1 = (rng.standard_normal(n) * 0.01).astype(np.float32)
    v1 = (rng.standard_normal(n) * 0.001).astype(np.float32)
    w2, v2 = w1.copy(), v1.copy()
    oracle_mod.sgd_momentum(a16, w1, v1, 0.01, 0.9, 5e-4)
    oracle_mod.sgd_momentum(a16.astype(np.float32), w2, v2, 0.01, 0.9, 5e-4)
    assert np.array_equal(w1.view(np.uint32), w2.view(np.uint32))
    assert np.array_equal(v1.view(np.uint32), v2.view(np.uint32))


def test_each_operation_is_rounded_separately_hand_cases(oracle_mod):
    """A fused multiply-add keeps the low bits of a product that separate rounding drops.  Two cancellations make
    those bits the whole result: (a) mu*v equal to the rounded lr*g, (b) g equal to minus the rounded wd*w."""
    lr, wd = np.float32(0.01), np.float32(5e-4)
    g = np.array([1.0 / 3.0], np.float32)
    lg = rn(fr(lr) * fr(g[0]))
    assert fr(lg) != fr(lr) * fr(g[0])                       # the product is inexact: the case discriminates
    w, v = np.zeros(1, np.float32), np.array([lg], np.float32)
    oracle_mod.sgd_momentum(g, w, v, float(lr), 1.0, 0.0)     # mv = lg exactly, so v' = lg - lg
    assert v[0] == 0.0 and w[0] == 0.0
    w0 = np.array([0.7], np.float32)
    dw = rn(fr(wd) * fr(w0[0]))
    assert fr(dw) != fr(wd) * fr(w0[0])
    w, v = w0.copy(), np.zeros(1, np.float32)
    oracle_mod.sgd_momentum(np.array([-dw], np.float32), w, v, float(lr), 0.0, float(wd))   # gg = -dw + dw
    assert v[0] == 0.0 and w[0] == w0[0]


def test_update_equals_exact_arithmetic_rounded_after_every_operation(oracle_mod):
    """Brute force: every product, sum and difference formed exactly (rationals) and rounded correctly to
    binary32 on its own, on values spread over many binades.  The same with any one product fused into the
    following sum must differ somewhere, or the inputs would not tell the two apart."""
    rng = np.random.default_rng(12)
    n = 400
    spread = lambda lo, hi: (np.exp2(rng.uniform(lo, hi, n)) * rng.choice([-1, 1], n)).astype(np.float32)
    g, w0, v0 = spread(-12, 2), spread(-8, 3), spread(-14, 0)
    lr, mu, wd = np.float32(0.01), np.float32(0.9), np.float32(5e-4)
    w, v = w0.copy(), v0.copy()
    oracle_mod.sgd_momentum(g, w, v, float(lr), float(mu), float(wd))
    fused_differs = [0, 0]
    for j in range(n):
        dw = rn(fr(wd) * fr(w0[j]))
        gg = rn(fr(g[j]) + fr(dw))
        mv = rn(fr(mu) * fr(v0[j]))
        lg = rn(fr(lr) * fr(gg))
        vn = rn(fr(mv) - fr(lg))
        wn = rn(fr(w0[j]) + fr(vn))
        assert v[j] == vn and w[j] == wn, j
        fused_differs[0] += rn(fr(mv) - fr(lr) * fr(gg)) != vn
        fused_differs[1] += rn(fr(g[j]) + fr(wd) * fr(w0[j])) != gg
    assert min(fused_differs) > 0, fused_differs


def test_easgd_equals_exact_arithmetic_rounded_after_every_operation(oracle_mod):
    rng = np.random.default_rng(13)
    n = 400
    spread = lambda lo, hi: (np.exp2(rng.uniform(lo, hi, n)) * rng.choice([-1, 1], n)).astype(np.float32)
    x0, c0 = spread(-8, 3), spread(-8, 3)
    alpha = np.float32(0.0625 * 1.7)                            # not a power of two: alpha * diff is inexact
    x, c = x0.copy(), c0.copy()
    oracle_mod.easgd(x, c, float(alpha))
    fused_differs = 0
    for j in range(n):
        diff = rn(fr(x0[j]) - fr(c0[j]))
        d = rn(fr(alpha) * fr(diff))
        assert x[j] == rn(fr(x0[j]) - fr(d)) and c[j] == rn(fr(c0[j]) + fr(d)), j
        fused_differs += rn(fr(x0[j]) - fr(alpha) * fr(diff)) != x[j]
    assert fused_differs > 0


# ---------------------------------------------------------------- elastic averaging

def test_easgd_conserves_sum_exactly_on_dyadic_grid(oracle_mod):
    """Inputs on multiples of 2^-10 in [-1, 1) and alpha = 2^-4: every operation
    is exact, so x' + c' == x + c bit for bit."""
    rng = np.random.default_rng(6)
    n = 50_000
    x = (rng.integers(-1024, 1024, n) / 1024.0).astype(np.float32)
    c = (rng.integers(-1024, 1024, n) / 1024.0).astype(np.float32)
    x0, c0 = x.copy(), c.copy()
    oracle_mod.easgd(x, c, 2.0 ** -4)
    assert np.array_equal(x + c, x0 + c0)
    assert np.array_equal(x, x0 - (x0 - c0) / 16)
    assert np.array_equal(c, c0 + (x0 - c0) / 16)
    assert np.any(x != x0)


def test_easgd_conserves_sum_over_k_workers(oracle_mod):
    rng = np.random.default_rng(7)
    n, k, alpha = 20_000, 8, 0.5 / 8
    xs = [(rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(k)]
    c = (rng.standard_normal(n) * 0.01).astype(np.float32)
    tot0 = np.sum(np.stack(xs + [c]).astype(np.float64), axis=0)
    for r in range(5):
        for i in rng.permutation(k):
            oracle_mod.easgd(xs[i], c, alpha)
    tot1 = np.sum(np.stack(xs + [c]).astype(np.float64), axis=0)
    assert np.max(np.abs(tot1 - tot0)) <= 40 * 2 * 2.0 ** -24 * 0.06


def test_easgd_half_rate_meets_at_midpoint(oracle_mod):
    rng = np.random.default_rng(8)
    n = 10_000
    x = (rng.integers(-1024, 1024, n) / 512.0).astype(np.float32)
    c = (rng.integers(-1024, 1024, n) / 512.0).astype(np.float32)
    mid = (x + c) / 2
    oracle_mod.easgd(x, c, 0.5)
    assert np.array_equal(x, mid) and np.array_equal(c, mid)


def test_easgd_gap_decays_geometrically(oracle_mod):
    """One pair repeated t times: x_t - c_t = (1 - 2 alpha)^t (x_0 - c_0)."""
    rng = np.random.default_rng(9)
    n, alpha, T = 5000, 0.0625, 30
    x = (rng.standard_normal(n) * 0.01).astype(np.float32)
    c = (rng.standard_normal(n) * 0.01).astype(np.float32)
    gap0 = x.astype(np.float64) - c.astype(np.float64)
    for _ in range(T):
        oracle_mod.easgd(x, c, alpha)
    want = (1 - 2 * alpha) ** T * gap0
    got = x.astype(np.float64) - c.astype(np.float64)
    assert np.max(np.abs(got - want)) <= 1e-5 * np.max(np.abs(gap0)) * (1 - 2 * alpha) ** T + 1e-8
    # direction: the worker moved toward the center, not away
    assert np.all(np.abs(got) <= np.abs(gap0))


def test_easgd_zero_rate_is_identity(oracle_mod):
    rng = np.random.default_rng(10)
    x = rng.standard_normal(1000).astype(np.float32)
    c = rng.standard_normal(1000).astype(np.float32)
    x0, c0 = x.copy(), c.copy()
    oracle_mod.easgd(x, c, 0.0)
    assert np.array_equal(x.view(np.uint32), x0.view(np.uint32))
    assert np.array_equal(c.view(np.uint32), c0.view(np.uint32))


# ---------------------------------------------------------------- diagnostics

def test_stats_against_numpy_and_exact_sum(oracle_mod):
    import math
    rng = np.random.default_rng(11)
    a = (rng.standard_normal(200_001) * 0.01).astype(np.float32)
    a[[5, 77, 1000]] = [np.inf, -np.inf, np.nan]
    a[123] = -3.5
    bad, mx, ss = oracle_mod.stats(a)
    fin = a[np.isfinite(a)].astype(np.float64)
    assert bad == 3 and mx == 3.5
    exact = math.fsum((fin * fin).tolist())        # squares of binary32 values are exact in binary64
    assert abs(ss - exact) <= 1e-12 * exact
    h = a.astype(np.float16)
    badh, mxh, ssh = oracle_mod.stats(h)
    finh = h[np.isfinite(h)].astype(np.float64)
    assert badh == 3 and mxh == 3.5
    assert abs(ssh - math.fsum((finh * finh).tolist())) <= 1e-12 * ssh


def test_stats_special_cases(oracle_mod):
    assert oracle_mod.stats(np.zeros(0, np.float32)) == (0, 0.0, 0.0)
    assert oracle_mod.stats(np.array([np.nan, np.inf], np.float32)) == (2, 0.0, 0.0)
    assert oracle_mod.stats(np.array([-0.0, 1e-45], np.float32)) == (0, float(np.float32(1e-45)), float(np.float32(1e-45)) ** 2)
    # an overflow in the pack shows up as one non-finite element
    g = np.array([1.0, 70000.0, -2.0], np.float32)
    assert oracle_mod.stats(oracle_mod.pack_fp16(g)) == (1, 2.0, 5.0)
    parts = [np.array([3.0, 4.0], np.float32), np.array([np.inf, -12.0], np.float32)]
    assert oracle_mod.stats_tensors(parts) == (1, 12.0, 169.0)
