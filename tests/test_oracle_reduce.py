"""Pins for the oracle's fixed-order sum and average (Section 3.2: the sum step
of Alltoall-sum-Allgather, at full precision; Section 4: averaging weights vs
summing updates)."""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from exact_arith import exact_round_f32


def f32(x):
    return np.asarray(x, dtype=np.float32)


def test_two_identical_buffers_give_exactly_twice(oracle_mod):
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100_000) * 0.01).astype(np.float32)
    s = oracle_mod.reduce_avg([x, x.copy()], mode=oracle_mod.SUM)
    assert np.array_equal(s, 2 * x)            # doubling is exact in binary32
    a = oracle_mod.reduce_avg([x, x.copy()])
    assert np.array_equal(a.view(np.uint32), x.view(np.uint32))   # idempotent


@pytest.mark.parametrize("k", [2, 4, 8, 16, 64])
def test_k_identical_half_valued_buffers(oracle_mod, k):
    """k*x is exactly representable at every partial sum when x has an 11-bit
    significand and k <= 2^13, so the sum is exact and the average returns x."""
    rng = np.random.default_rng(k)
    x16 = (rng.standard_normal(50_000) * 0.01).astype(np.float16)
    x = x16.astype(np.float32)
    s = oracle_mod.reduce_avg([x] * k, mode=oracle_mod.SUM)
    assert np.array_equal(s, np.float32(k) * x)
    a = oracle_mod.reduce_avg([x16] * k, out_dtype=np.float16)
    assert np.array_equal(a.view(np.uint16), x16.view(np.uint16))
    a32 = oracle_mod.reduce_avg([x16] * k, out_dtype=np.float32)
    assert np.array_equal(a32.view(np.uint32), x.view(np.uint32))


def test_order_sensitive_hand_cases(oracle_mod):
    """2^24 + 1 is a tie in binary32 and rounds to 2^24 (even), so the position
    of the cancelling term decides the result."""
    big, one = 2.0 ** 24, 1.0
    r = oracle_mod.reduce_avg([f32([big]), f32([one]), f32([-big])], mode=oracle_mod.SUM)
    assert r[0] == 0.0
    r = oracle_mod.reduce_avg([f32([big]), f32([-big]), f32([one])], mode=oracle_mod.SUM)
    assert r[0] == 1.0
    r = oracle_mod.reduce_avg([f32([one]), f32([big]), f32([-big])], mode=oracle_mod.SUM)
    assert r[0] == 0.0
    # 2^24 + 3 = tie between 2^24+2 and 2^24+4 -> even significand -> 2^24+4
    r = oracle_mod.reduce_avg([f32([big]), f32([3.0]), f32([-big])], mode=oracle_mod.SUM)
    assert r[0] == 4.0
    # four workers, left fold: ((1e8 + 1) + 1) + -1e8 = 0, but ((1 + 1) + 1e8) - 1e8 = 0 too;
    # (1 + 1 + 1 + 1 ...) first reaches the ulp: use ulp(1e8) = 8
    c = [f32([1e8])] + [f32([3.0])] * 3 + [f32([-1e8])]
    # 1e8 + 3 -> 1e8 (3 < 4 = half ulp) three times, then - 1e8 = 0
    assert oracle_mod.reduce_avg(c, mode=oracle_mod.SUM)[0] == 0.0
    c = [f32([3.0])] * 3 + [f32([1e8]), f32([-1e8])]
    # 9 + 1e8 -> 1e8 + 8, minus 1e8 = 8
    assert oracle_mod.reduce_avg(c, mode=oracle_mod.SUM)[0] == 8.0


def test_order_sensitive_hand_cases_with_half_contributions(oracle_mod):
    """The same for binary16 contributions, which are widened exactly and summed in binary32: 65504 (the largest
    half) has ulp 2^-8 in binary32, so adding 2^-10 to it is lost, while 2^-10 survives next to zero."""
    big, small = np.float16(65504.0), np.float16(2.0 ** -10)
    h = lambda x: np.array([x], np.float16)
    r = oracle_mod.reduce_avg([h(big), h(-big), h(small)], mode=oracle_mod.SUM)
    assert r[0] == np.float32(2.0 ** -10)
    r = oracle_mod.reduce_avg([h(big), h(small), h(-big)], mode=oracle_mod.SUM)
    assert r[0] == 0.0
    r = oracle_mod.reduce_avg([h(small), h(big), h(-big)], mode=oracle_mod.SUM)
    assert r[0] == 0.0
    # three quarters of an ulp, added one at a time: each 3 * 2^-10 alone rounds away, together they would not
    c = [h(big)] + [h(np.float16(3 * 2.0 ** -10))] * 3 + [h(-big)]
    assert oracle_mod.reduce_avg(c, mode=oracle_mod.SUM)[0] == 2.0 ** -8 * 3   # each step rounds up one ulp
    c = [h(np.float16(3 * 2.0 ** -10))] * 3 + [h(big), h(-big)]
    assert oracle_mod.reduce_avg(c, mode=oracle_mod.SUM)[0] == 2.0 ** -8 * 2   # 9 * 2^-10 rounds to two ulps
    # the result as binary16, and the average, go through the same fold
    r = oracle_mod.reduce_avg([h(big), h(-big), h(small), h(small)], np.float16, oracle_mod.AVG)
    assert r.dtype == np.float16 and r[0] == np.float16(2.0 ** -11)


def test_running_sum_starts_from_first_contribution(oracle_mod):
    nz, pz = f32([-0.0]), f32([0.0])
    assert np.signbit(oracle_mod.reduce_avg([nz])[0])
    assert np.signbit(oracle_mod.reduce_avg([nz, nz.copy()])[0])
    assert not np.signbit(oracle_mod.reduce_avg([nz, pz])[0])
    assert np.signbit(oracle_mod.reduce_avg([nz], mode=oracle_mod.SUM)[0])


def test_left_fold_matches_exact_fold_step_by_step(oracle_mod):
    """Brute force: fold with exact rationals, rounding each partial sum
    correctly to binary32, on values spread over many binades."""
    rng = np.random.default_rng(5)
    k, n = 8, 300
    cs = [(np.exp2(rng.uniform(-20, 20, n)) * rng.choice([-1, 1], n)).astype(np.float32)
          for _ in range(k)]
    got = oracle_mod.reduce_avg(cs, mode=oracle_mod.SUM)
    for j in range(n):
        s = cs[0][j]
        for i in range(1, k):
            s = exact_round_f32(Fraction(float(s)) + Fraction(float(cs[i][j])))
        assert got[j] == s, j
    # and it must differ from the reversed order somewhere (order matters here)
    rev = oracle_mod.reduce_avg(cs[::-1], mode=oracle_mod.SUM)
    assert np.any(got != rev)


@pytest.mark.parametrize("k", [2, 3, 5, 7, 8, 12])
def test_average_is_one_correctly_rounded_division(oracle_mod, k):
    rng = np.random.default_rng(100 + k)
    n = 200
    cs = [(rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(k)]
    s = oracle_mod.reduce_avg(cs, mode=oracle_mod.SUM)
    a = oracle_mod.reduce_avg(cs)
    for j in range(n):
        assert a[j] == exact_round_f32(Fraction(float(s[j])) / k), (k, j)


def test_sum_within_forward_error_bound_of_exact(oracle_mod):
    """|s32 - exact| <= (k-1) * 2^-24 * max |partial sum| (one half-ulp per add)."""
    rng = np.random.default_rng(9)
    k, n = 8, 200_000
    cs = [(rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(k)]
    got = oracle_mod.reduce_avg(cs, mode=oracle_mod.SUM).astype(np.float64)
    part = np.cumsum(np.stack(cs).astype(np.float64), axis=0)     # exact to ~2^-50
    bound = (k - 1) * 2.0 ** -24 * np.abs(part).max(axis=0) * (1 + 1e-6)
    assert np.all(np.abs(got - part[-1]) <= bound)


def test_half_valued_gradients_sum_exactly(oracle_mod):
    """Eight sigma = 0.01 halves: every order gives the exact sum in binary32,
    so the benchmark's own data cannot see a wrong order; wide-range halves can."""
    rng = np.random.default_rng(13)
    k, n = 8, 200_000
    hs = [(rng.standard_normal(n) * 0.01).astype(np.float16) for _ in range(k)]
    got = oracle_mod.reduce_avg(hs, out_dtype=np.float32, mode=oracle_mod.SUM)
    exact = np.sum(np.stack(hs).astype(np.float64), axis=0)
    assert np.mean(got.astype(np.float64) == exact) > 0.999
    wide = [wl.wide_range_halves([n], 77, i)[0].astype(np.float16) for i in range(k)]
    fwd = oracle_mod.reduce_avg(wide, out_dtype=np.float32, mode=oracle_mod.SUM)
    rev = oracle_mod.reduce_avg(wide[::-1], out_dtype=np.float32, mode=oracle_mod.SUM)
    assert np.mean(fwd != rev) > 0.01


def test_half_output_is_one_rne_of_the_float_average(oracle_mod):
    rng = np.random.default_rng(17)
    k, n = 8, 100_000
    hs = [(rng.standard_normal(n) * 0.01).astype(np.float16) for _ in range(k)]
    a32 = oracle_mod.reduce_avg(hs, out_dtype=np.float32)
    a16 = oracle_mod.reduce_avg(hs, out_dtype=np.float16)
    # numpy's cast is the library RNE; the oracle's own cast is pinned elsewhere
    assert np.array_equal(a16.view(np.uint16), a32.astype(np.float16).view(np.uint16))
    # and the float average equals the exact mean here (exact sum, k a power of two)
    exact = np.mean(np.stack(hs).astype(np.float64), axis=0)
    ok = np.abs(exact) >= 2.0 ** -126
    assert np.array_equal(a32.astype(np.float64)[ok], exact[ok])


def test_weight_averaging_equals_summed_updates(oracle_mod):
    """Section 4: averaging weights after each worker's own step with the
    learning rate scaled by k equals one step on the summed updates:
    mean_i (w - k lr g_i) = w - lr sum_i g_i, up to rounding."""
    rng = np.random.default_rng(21)
    k, n, lr = 8, 50_000, 0.01
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    gs = [(rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(k)]
    # AWAGD: each worker descends alone (mu = 0), then weights are averaged
    ws = []
    for g in gs:
        wi, vi = w.copy(), np.zeros(n, np.float32)
        oracle_mod.sgd_momentum(g, wi, vi, k * lr, 0.0, 0.0)
        ws.append(wi)
    awagd = oracle_mod.reduce_avg(ws)
    # SUBGD: sum the updates, then one descent step with the unscaled rate
    gsum = oracle_mod.reduce_avg(gs, mode=oracle_mod.SUM)
    w2, v2 = w.copy(), np.zeros(n, np.float32)
    oracle_mod.sgd_momentum(gsum, w2, v2, lr, 0.0, 0.0)
    assert np.max(np.abs(awagd - w2)) <= 4e-7 * np.max(np.abs(w)) + 1e-8
    assert np.max(np.abs(w2 - w)) > 1e-4        # the step actually moved


def test_argument_errors(oracle_mod):
    x = np.zeros(4, np.float32)
    with pytest.raises(ValueError):
        oracle_mod.reduce_avg([])
    with pytest.raises(ValueError):
        oracle_mod.reduce_avg([x, np.zeros(5, np.float32)])
    with pytest.raises(TypeError):
        oracle_mod.reduce_avg([x, np.zeros(4, np.float16)])
