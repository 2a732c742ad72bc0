"""GPU parity: every libpxchg call against the CPU oracle, element by element, on
shapes that span several chunks, ragged tails, tiny tensors and misaligned
pointers.  Bit-exact for the binary16 conversion and the fixed-order sums; the
updates are compared bit-exactly too (both sides round every operation to
binary32), which is stricter than the stated 1e-6 tolerance."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import (assert_bits_equal, assert_close_params, empty_like_device, to_device,
                      to_host)

pytestmark = pytest.mark.gpu

# several full chunks + ragged tails + tiny tensors + an empty one
RAGGED = [1, 3, 63, 64, 65, 0, 8 * 1000 + 1, 20_000, 2 * 8192 + 5, 8192, 8191, 70_001]


@pytest.fixture(scope="module")
def px():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1605_08325_amd as px
    px.load()
    return px


def _gauss(counts, seed, worker=0, sigma=0.01, role="grad"):
    return [a.copy() for a in wl.gaussian_tensors(counts, sigma, seed, role, worker)]


# ------------------------------------------------------------------ pack / unpack

def test_unpack_all_halves_then_pack_back(px, oracle_mod):
    hs = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16).view(np.float16)
    table = px.Table([hs.size])
    d_h = to_device([hs])
    d_w = empty_like_device([hs.size], np.float32)
    d_b = empty_like_device([hs.size], np.float16)
    sh, sw, sb = table.bufset(d_h), table.bufset(d_w), table.bufset(d_b)
    px.unpack_fp16(table, [sh], [sw])
    px.pack_fp16(table, [sw], [sb])
    wide = to_host(d_w)
    assert_bits_equal(wide, [oracle_mod.unpack_fp16(hs)], "unpack", nan_as_class=True)
    back = to_host(d_b)
    assert_bits_equal(back, [oracle_mod.pack_fp16(oracle_mod.unpack_fp16(hs))], "round trip",
                      nan_as_class=True)
    # NaN keeps its sign through both directions
    nan = np.isnan(hs)
    assert np.array_equal(back[0].view(np.uint16)[nan] & 0x8000, hs.view(np.uint16)[nan] & 0x8000)


def test_pack_ties_and_boundaries(px, oracle_mod):
    lo = np.arange(0, 0x7C00, dtype=np.uint32).astype(np.uint16).view(np.float16).astype(np.float64)
    hi = np.append(lo[1:], 65536.0)
    mid = ((lo + hi) / 2).astype(np.float32)
    vals = np.concatenate([
        mid, np.nextafter(mid, np.float32(-np.inf)), np.nextafter(mid, np.float32(np.inf)),
        np.array([65504.0, 65519.996, 65520.0, 65536.0, 3e38, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25,
                  2.0 ** -26, 0.0, 1e-45, 1.1754942e-38, np.inf], np.float32)])
    vals = np.concatenate([vals, -vals]).astype(np.float32)
    table = px.Table([vals.size])
    d_in = to_device([vals])
    d_out = empty_like_device([vals.size], np.float16)
    px.pack_fp16(table, [table.bufset(d_in)], [table.bufset(d_out)])
    assert_bits_equal(to_host(d_out), [oracle_mod.pack_fp16(vals)], "ties and boundaries")


def test_pack_random_bit_patterns(px, oracle_mod):
    rng = np.random.default_rng(11)
    x = rng.integers(0, 1 << 32, 6_000_001, dtype=np.uint64).astype(np.uint32).view(np.float32)
    table = px.Table([x.size])
    d_in = to_device([x])
    d_out = empty_like_device([x.size], np.float16)
    px.pack_fp16(table, [table.bufset(d_in)], [table.bufset(d_out)])
    assert_bits_equal(to_host(d_out), [oracle_mod.pack_fp16(x)], "random bits", nan_as_class=True)


@pytest.mark.parametrize("offset", [0, 1, 3])
def test_pack_many_workers_ragged(px, oracle_mod, offset):
    k = 5
    table = px.Table(RAGGED)
    src = [_gauss(RAGGED, 100 + offset, w) for w in range(k)]
    d_src = [to_device(s, offset) for s in src]
    d_dst = [empty_like_device(RAGGED, np.float16, offset, fill=7.0) for _ in range(k)]
    px.pack_fp16(table, [table.bufset(s) for s in d_src], [table.bufset(d) for d in d_dst])
    for w in range(k):
        assert_bits_equal(to_host(d_dst[w]), oracle_mod.pack_fp16_tensors(src[w]), f"worker {w}")
    # nothing outside the tensors was written (guard elements keep their fill)
    for w in range(k):
        for t in d_dst[w]:
            base = t._base if t._base is not None else t
            host = base.cpu().numpy()
            assert np.all(host[:offset] == 7.0) and np.all(host[offset + t.numel():] == 7.0)


def test_pack_mixed_alignment_uses_elementwise_path(px, oracle_mod):
    """Source 4 bytes off, destination 16-byte aligned: no common vector alignment."""
    counts = [5000, 17, 8192 + 3]
    table = px.Table(counts)
    src = _gauss(counts, 42)
    d_src = to_device(src, 1)
    d_dst = empty_like_device(counts, np.float16, 0)
    px.pack_fp16(table, [table.bufset(d_src)], [table.bufset(d_dst)])
    assert_bits_equal(to_host(d_dst), oracle_mod.pack_fp16_tensors(src), "mixed alignment")
    d_dst2 = empty_like_device(counts, np.float16, 2)     # 4-byte offset on the half side
    px.pack_fp16(table, [table.bufset(d_src)], [table.bufset(d_dst2)])
    assert_bits_equal(to_host(d_dst2), oracle_mod.pack_fp16_tensors(src), "mixed alignment 2")


# ------------------------------------------------------------------ reduce + average

@pytest.mark.parametrize("k", [1, 2, 3, 5, 8, 9, 13, 16, 64])
@pytest.mark.parametrize("in_dt,out_dt", [(np.float32, np.float32), (np.float16, np.float16),
                                          (np.float16, np.float32), (np.float32, np.float16)])
def test_reduce_avg_ragged(px, oracle_mod, k, in_dt, out_dt):
    counts = RAGGED if k <= 16 else [1, 65, 8192 + 9, 3000]
    table = px.Table(counts)
    contrib = []
    for w in range(k):
        g = _gauss(counts, 200 + k, w)
        contrib.append([a.astype(in_dt) for a in g])
    d_c = [to_device(c) for c in contrib]
    sets = [table.bufset(c) for c in d_c]
    for mode in (px.AVG, px.SUM):
        d_out = empty_like_device(counts, out_dt)
        px.reduce_avg(table, sets, table.bufset(d_out), mode)
        want = oracle_mod.reduce_avg_tensors(contrib, out_dt, mode)
        assert_bits_equal(to_host(d_out), want, f"k={k} mode={mode}")


@pytest.mark.parametrize("offset", [1, 2])
def test_reduce_avg_misaligned(px, oracle_mod, offset):
    k = 8
    table = px.Table(RAGGED)
    contrib = [[a.astype(np.float16) for a in _gauss(RAGGED, 300, w)] for w in range(k)]
    d_c = [to_device(c, offset) for c in contrib]
    d_out = empty_like_device(RAGGED, np.float16, offset)
    px.reduce_avg(table, [table.bufset(c) for c in d_c], table.bufset(d_out))
    assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(contrib, np.float16), "misaligned")


def test_reduce_order_sensitive_float32(px, oracle_mod):
    """k = 8, binary32 transfer: the sequential order is visible in the last bit."""
    k, counts = 8, [100_003, 8192 * 3 + 1]
    table = px.Table(counts)
    contrib = [_gauss(counts, 400, w) for w in range(k)]
    d_c = [to_device(c) for c in contrib]
    d_out = empty_like_device(counts, np.float32)
    px.reduce_avg(table, [table.bufset(c) for c in d_c], table.bufset(d_out))
    got = to_host(d_out)
    assert_bits_equal(got, oracle_mod.reduce_avg_tensors(contrib), "fp32 order")
    rev = oracle_mod.reduce_avg_tensors(contrib[::-1])
    assert np.mean(got[0] != rev[0]) > 0.05          # a reversed order would be caught


def test_reduce_order_sensitive_wide_range_halves(px, oracle_mod):
    k, counts = 8, [100_003, 8192 * 3 + 1]
    table = px.Table(counts)
    contrib = [[a.astype(np.float16) for a in wl.wide_range_halves(counts, 500, w)] for w in range(k)]
    d_c = [to_device(c) for c in contrib]
    for out_dt in (np.float32, np.float16):
        d_out = empty_like_device(counts, out_dt)
        px.reduce_avg(table, [table.bufset(c) for c in d_c], table.bufset(d_out), px.SUM)
        got = to_host(d_out)
        assert_bits_equal(got, oracle_mod.reduce_avg_tensors(contrib, out_dt, px.SUM), "wide halves")
    rev = oracle_mod.reduce_avg_tensors(contrib[::-1], np.float32, px.SUM)
    d_out = empty_like_device(counts, np.float32)
    px.reduce_avg(table, [table.bufset(c) for c in d_c], table.bufset(d_out), px.SUM)
    assert np.mean(to_host(d_out)[0] != rev[0]) > 0.01


def test_reduce_special_values(px, oracle_mod):
    """Signed zeros, infinities, NaN, subnormals: s starts from the first contribution."""
    sp = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 1.1754942e-38, 3e38, -3e38,
                   65504.0, 2.0 ** -24, 2.0 ** -25, 1.0], np.float32)
    a = np.repeat(sp, sp.size)
    b = np.tile(sp, sp.size)
    table = px.Table([a.size])
    for k_extra in (0, 1):
        contrib = [[a], [b]] + [[np.full_like(a, -0.0)]] * k_extra
        d_c = [to_device(c) for c in contrib]
        for out_dt in (np.float32, np.float16):
            for mode in (px.AVG, px.SUM):
                d_out = empty_like_device([a.size], out_dt)
                px.reduce_avg(table, [table.bufset(c) for c in d_c], table.bufset(d_out), mode)
                assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(contrib, out_dt, mode),
                                  f"special k={2 + k_extra}", nan_as_class=True)
    # k = 1: a lone -0 stays -0
    d_c = to_device([a])
    d_out = empty_like_device([a.size], np.float32)
    px.reduce_avg(table, [table.bufset(d_c)], table.bufset(d_out))
    assert_bits_equal(to_host(d_out), [oracle_mod.reduce_avg([a])], "k=1", nan_as_class=True)


@pytest.mark.parametrize("dt", [np.float32, np.float16])
@pytest.mark.parametrize("k", [2, 4, 8, 9])
@pytest.mark.parametrize("which", ["first", "last", "middle"])
def test_reduce_in_place_into_one_of_the_contributions(px, oracle_mod, dt, k, which):
    """Weight averaging writes the mean back over one worker's copy: the output may be any of the contributions
    (every lane reads all k values of its elements before it stores), float32 or binary16, every kernel shape."""
    counts = [10_000, 33, 0, 70_001, 8192 * 3]
    table = px.Table(counts)
    contrib = [[a.astype(dt) for a in _gauss(counts, 600 + k, w, role="param")] for w in range(k)]
    want = oracle_mod.reduce_avg_tensors(contrib, dt)
    d_c = [to_device(c) for c in contrib]
    sets = [table.bufset(c) for c in d_c]
    target = {"first": 0, "last": k - 1, "middle": k // 2}[which]
    px.reduce_avg(table, sets, sets[target])
    assert_bits_equal(to_host(d_c[target]), want, f"in place into contribution {target}")
    for w in range(k):                                      # the others are untouched
        if w != target:
            assert_bits_equal(to_host(d_c[w]), contrib[w], f"contribution {w}")


# ------------------------------------------------------------------ momentum SGD

@pytest.mark.parametrize("g_dt", [np.float32, np.float16])
@pytest.mark.parametrize("wd", [0.0, 5e-4])
@pytest.mark.parametrize("offset", [0, 1])
def test_sgd_momentum_steps(px, oracle_mod, g_dt, wd, offset):
    table = px.Table(RAGGED)
    w = _gauss(RAGGED, 700, role="param")
    v = _gauss(RAGGED, 701, sigma=1e-3, role="velocity")
    d_w, d_v = to_device(w, offset), to_device(v, offset)
    sw, sv = table.bufset(d_w), table.bufset(d_v)
    g_off = offset                                      # same element offset: a common head exists
    for step in range(3):
        g = [a.astype(g_dt) for a in _gauss(RAGGED, 702, worker=step)]
        d_g = to_device(g, g_off)
        px.sgd_momentum(table, table.bufset(d_g), sw, sv, 0.01, 0.9, wd)
        oracle_mod.sgd_momentum_tensors(g, w, v, 0.01, 0.9, wd)
        assert_bits_equal(to_host(d_w), w, f"w step {step}")
        assert_bits_equal(to_host(d_v), v, f"v step {step}")
    assert_close_params(to_host(d_w), w)


def test_sgd_momentum_operands_without_common_alignment(px, oracle_mod):
    counts = [8192 + 77, 5]
    table = px.Table(counts)
    w, v, g = _gauss(counts, 710, role="param"), _gauss(counts, 711, role="velocity"), _gauss(counts, 712)
    d_w, d_v, d_g = to_device(w, 1), to_device(v, 0), to_device(g, 2)
    px.sgd_momentum(table, table.bufset(d_g), table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4)
    oracle_mod.sgd_momentum_tensors(g, w, v, 0.01, 0.9, 5e-4)
    assert_bits_equal(to_host(d_w), w, "w")
    assert_bits_equal(to_host(d_v), v, "v")


def test_sgd_momentum_tiny_values_keep_subnormals(px, oracle_mod):
    counts = [4099]
    rng = np.random.default_rng(8)
    w = [(rng.standard_normal(counts[0]) * 1e-38).astype(np.float32)]
    v = [(rng.standard_normal(counts[0]) * 1e-39).astype(np.float32)]
    g = [(rng.standard_normal(counts[0]) * 1e-37).astype(np.float32)]
    table = px.Table(counts)
    d_w, d_v, d_g = to_device(w), to_device(v), to_device(g)
    px.sgd_momentum(table, table.bufset(d_g), table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4)
    oracle_mod.sgd_momentum_tensors(g, w, v, 0.01, 0.9, 5e-4)
    assert_bits_equal(to_host(d_w), w, "subnormal w")
    assert_bits_equal(to_host(d_v), v, "subnormal v")
    assert np.any((np.abs(v[0]) < 1.1754944e-38) & (v[0] != 0))     # subnormals did occur


def test_update_and_elastic_special_values(px, oracle_mod):
    """Infinities, NaN, signed zeros, subnormals and the extremes of the range through the update (staged and
    fused) and the elastic step: the same bits as the oracle, NaN compared as a class (Inf - Inf, 0 * Inf)."""
    sp = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 1.1754942e-38, 3e38, -3e38, 1.0, -2.5],
                  np.float32)
    m = sp.size
    g = [np.repeat(sp, m * m)]
    w0 = [np.tile(np.repeat(sp, m), m)]
    v0 = [np.tile(sp, m * m)]
    n = g[0].size
    table = px.Table([n])
    for lr, mu, wd in ((0.01, 0.9, 5e-4), (0.0, 0.0, 0.0), (1.0, 1.0, 0.0)):
        w, v = [w0[0].copy()], [v0[0].copy()]
        d_w, d_v = to_device(w), to_device(v)
        px.sgd_momentum(table, table.bufset(to_device(g)), table.bufset(d_w), table.bufset(d_v), lr, mu, wd)
        oracle_mod.sgd_momentum_tensors(g, w, v, lr, mu, wd)
        assert_bits_equal(to_host(d_w), w, f"w lr={lr}", nan_as_class=True)
        assert_bits_equal(to_host(d_v), v, f"v lr={lr}", nan_as_class=True)
        # fused, two workers: the mean of (g, g) is g wherever 2g does not overflow; the oracle decides
        w2, v2 = [w0[0].copy()], [v0[0].copy()]
        d_w2, d_v2 = to_device(w2), to_device(v2)
        sets = [table.bufset(to_device(g)), table.bufset(to_device(g))]
        px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w2), table.bufset(d_v2), lr, mu, wd)
        oracle_mod.sgd_momentum_tensors(oracle_mod.reduce_avg_tensors([g, g]), w2, v2, lr, mu, wd)
        assert_bits_equal(to_host(d_w2), w2, f"fused w lr={lr}", nan_as_class=True)
        assert_bits_equal(to_host(d_v2), v2, f"fused v lr={lr}", nan_as_class=True)
    for alpha in (0.0625, 0.0, 0.5, 1.0):
        x, c = [w0[0].copy()], [v0[0].copy()]
        d_x, d_c = to_device(x), to_device(c)
        px.easgd(table, table.bufset(d_x), table.bufset(d_c), alpha)
        oracle_mod.easgd_tensors(x, c, alpha)
        assert_bits_equal(to_host(d_x), x, f"x alpha={alpha}", nan_as_class=True)
        assert_bits_equal(to_host(d_c), c, f"c alpha={alpha}", nan_as_class=True)


# ------------------------------------------------------------------ fused reduce + update

@pytest.mark.parametrize("k", [1, 2, 3, 8, 9, 13, 64])
@pytest.mark.parametrize("in_dt", [np.float32, np.float16])
@pytest.mark.parametrize("wire", ["f32", "f16"])
def test_fused_reduce_update_equals_two_calls_and_oracle(px, oracle_mod, k, in_dt, wire):
    table = px.Table(RAGGED)
    contrib = [[a.astype(in_dt) for a in _gauss(RAGGED, 800 + k, w)] for w in range(k)]
    w0 = _gauss(RAGGED, 801, role="param")
    v0 = _gauss(RAGGED, 802, sigma=1e-3, role="velocity")
    wire_np = np.float16 if wire == "f16" else np.float32
    wire_px = px.F16 if wire == "f16" else px.F32
    sets = [table.bufset(to_device(c)) for c in contrib]
    # oracle: two steps
    w_o, v_o = [a.copy() for a in w0], [a.copy() for a in v0]
    avg = oracle_mod.reduce_avg_tensors(contrib, wire_np)
    oracle_mod.sgd_momentum_tensors(avg, w_o, v_o, 0.01, 0.9, 5e-4)
    # GPU: two calls
    d_w2, d_v2 = to_device(w0), to_device(v0)
    d_avg = empty_like_device(RAGGED, wire_np)
    s_avg = table.bufset(d_avg)
    px.reduce_avg(table, sets, s_avg)
    px.sgd_momentum(table, s_avg, table.bufset(d_w2), table.bufset(d_v2), 0.01, 0.9, 5e-4)
    # GPU: fused
    d_w1, d_v1 = to_device(w0), to_device(v0)
    px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w1), table.bufset(d_v1), 0.01, 0.9, 5e-4,
                               px.AVG, wire_px)
    assert_bits_equal(to_host(d_w1), w_o, "fused w vs oracle")
    assert_bits_equal(to_host(d_v1), v_o, "fused v vs oracle")
    assert_bits_equal(to_host(d_w2), w_o, "two-call w vs oracle")
    assert_bits_equal(to_host(d_v2), v_o, "two-call v vs oracle")


# ------------------------------------------------------------------ elastic averaging

@pytest.mark.parametrize("offset", [0, 1])
def test_easgd_pair(px, oracle_mod, offset):
    table = px.Table(RAGGED)
    x = _gauss(RAGGED, 900, role="worker")
    c = _gauss(RAGGED, 901, role="center")
    d_x, d_c = to_device(x, offset), to_device(c, offset)
    sx, sc = table.bufset(d_x), table.bufset(d_c)
    for _ in range(3):
        px.easgd(table, sx, sc, 0.0625)
        oracle_mod.easgd_tensors(x, c, 0.0625)
    assert_bits_equal(to_host(d_x), x, "x")
    assert_bits_equal(to_host(d_c), c, "c")


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8, 11])
@pytest.mark.parametrize("in_dt", [np.float32, np.float16])
@pytest.mark.parametrize("offsets", [(1, 1, 1), (2, 2, 2), (2, 1, 1), (0, 1, 0)])
def test_fused_reduce_update_misaligned(px, oracle_mod, k, in_dt, offsets):
    """Every lane width of the fused kernel (by k and contribution type) with operands that are off 16-byte
    alignment by the same number of elements (head, vector body, tail), by the same number of bytes, or
    without a common alignment (element-wise path)."""
    oc, ow, ov = offsets
    table = px.Table(RAGGED)
    contrib = [[a.astype(in_dt) for a in _gauss(RAGGED, 820 + k, w)] for w in range(k)]
    w_o = _gauss(RAGGED, 821, role="param")
    v_o = _gauss(RAGGED, 822, sigma=1e-3, role="velocity")
    d_w, d_v = to_device(w_o, ow), to_device(v_o, ov)
    sets = [table.bufset(to_device(c, oc)) for c in contrib]
    px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4, px.AVG, px.F16)
    avg = oracle_mod.reduce_avg_tensors(contrib, np.float16)
    oracle_mod.sgd_momentum_tensors(avg, w_o, v_o, 0.01, 0.9, 5e-4)
    assert_bits_equal(to_host(d_w), w_o, "w")
    assert_bits_equal(to_host(d_v), v_o, "v")


@pytest.mark.parametrize("k,offset", [(2, 1), (3, 1), (4, 3), (8, 1), (8, 2)])
def test_easgd_round_misaligned(px, oracle_mod, k, offset):
    table = px.Table(RAGGED)
    xs = [_gauss(RAGGED, 930, w, role="worker") for w in range(k)]
    c = _gauss(RAGGED, 931, role="center")
    d_xs = [to_device(x, offset) for x in xs]
    d_c = to_device(c, offset if k != 3 else 0)      # k = 3: no common alignment
    px.easgd_round(table, [table.bufset(x) for x in d_xs], table.bufset(d_c), 0.0625)
    for i in range(k):
        oracle_mod.easgd_tensors(xs[i], c, np.float32(0.0625))
    for i in range(k):
        assert_bits_equal(to_host(d_xs[i]), xs[i], f"x[{i}]")
    assert_bits_equal(to_host(d_c), c, "center")


@pytest.mark.parametrize("k", [1, 2, 5, 8, 11])
def test_easgd_round_equals_k_pairs_in_order(px, oracle_mod, k):
    counts = RAGGED
    table = px.Table(counts)
    xs = [_gauss(counts, 910, w, role="worker") for w in range(k)]
    c = _gauss(counts, 911, role="center")
    d_xs = [to_device(x) for x in xs]
    d_c = to_device(c)
    sets = [table.bufset(x) for x in d_xs]
    sc = table.bufset(d_c)
    orders = wl.worker_orders(912, k, 4)
    for order in orders:
        px.easgd_round(table, [sets[i] for i in order], sc, 0.5 / k)
        for i in order:
            oracle_mod.easgd_tensors(xs[i], c, np.float32(0.5 / k))
    for i in range(k):
        assert_bits_equal(to_host(d_xs[i]), xs[i], f"x[{i}]")
    assert_bits_equal(to_host(d_c), c, "center")
    # the order matters: a fixed order gives a different center
    if k >= 5:
        xs2 = [_gauss(counts, 910, w, role="worker") for w in range(k)]
        c2 = _gauss(counts, 911, role="center")
        for _ in orders:
            for i in range(k):
                oracle_mod.easgd_tensors(xs2[i], c2, np.float32(0.5 / k))
        assert any(np.any(a != b) for a, b in zip(c, c2))


# ------------------------------------------------------------------ launch shapes

@pytest.mark.parametrize("chunk,bpc", [(512, 1), (1024, 0), (2048, 0), (32768, 0), (8192, 2), (4096, 8)])
def test_results_do_not_depend_on_launch_shape(px, oracle_mod, chunk, bpc):
    old = (px.get_option(px.OPT_CHUNK_ELEMS), px.get_option(px.OPT_BLOCKS_PER_CU))
    try:
        px.set_option(px.OPT_CHUNK_ELEMS, chunk)
        px.set_option(px.OPT_BLOCKS_PER_CU, bpc)
        k = 8
        table = px.Table(RAGGED)
        contrib = [[a.astype(np.float16) for a in _gauss(RAGGED, 950, w)] for w in range(k)]
        sets = [table.bufset(to_device(c)) for c in contrib]
        d_out = empty_like_device(RAGGED, np.float16)
        px.reduce_avg(table, sets, table.bufset(d_out))
        assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(contrib, np.float16), "launch shape")
        src = [_gauss(RAGGED, 951, w) for w in range(3)]
        d_dst = [empty_like_device(RAGGED, np.float16) for _ in range(3)]
        px.pack_fp16(table, [table.bufset(to_device(s)) for s in src], [table.bufset(d) for d in d_dst])
        for w in range(3):
            assert_bits_equal(to_host(d_dst[w]), oracle_mod.pack_fp16_tensors(src[w]), "pack launch shape")
        # the in-place float32 kernels (two wavefronts of 4-element lanes) under the same launch shapes
        avg = oracle_mod.reduce_avg_tensors(contrib, np.float16)
        w_, v_ = _gauss(RAGGED, 952, role="param"), _gauss(RAGGED, 953, sigma=1e-3, role="velocity")
        d_w, d_v = to_device(w_), to_device(v_)
        px.sgd_momentum(table, table.bufset(d_out), table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4)
        oracle_mod.sgd_momentum_tensors(avg, w_, v_, 0.01, 0.9, 5e-4)
        assert_bits_equal(to_host(d_w), w_, "update launch shape")
        assert_bits_equal(to_host(d_v), v_, "update launch shape")
        x_, c_ = _gauss(RAGGED, 954, role="worker"), _gauss(RAGGED, 955, role="center")
        d_x, d_c = to_device(x_), to_device(c_)
        px.easgd(table, table.bufset(d_x), table.bufset(d_c), 0.0625)
        px.easgd_round(table, [table.bufset(d_w), table.bufset(d_v)], table.bufset(d_c), 0.0625)
        oracle_mod.easgd_tensors(x_, c_, 0.0625)
        oracle_mod.easgd_tensors(w_, c_, 0.0625)
        oracle_mod.easgd_tensors(v_, c_, 0.0625)
        assert_bits_equal(to_host(d_x), x_, "elastic launch shape")
        assert_bits_equal(to_host(d_c), c_, "elastic launch shape")
        assert_bits_equal(to_host(d_w), w_, "elastic round launch shape")
        # the kernels that run two workgroups per chunk: fused reduce+update of 8, elastic round of 5
        w2, v2 = _gauss(RAGGED, 956, role="param"), _gauss(RAGGED, 957, sigma=1e-3, role="velocity")
        d_w2, d_v2 = to_device(w2), to_device(v2)
        px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w2), table.bufset(d_v2), 0.01, 0.9, 5e-4, wire_dtype=px.F16)
        oracle_mod.sgd_momentum_tensors(avg, w2, v2, 0.01, 0.9, 5e-4)
        assert_bits_equal(to_host(d_w2), w2, "fused launch shape")
        assert_bits_equal(to_host(d_v2), v2, "fused launch shape")
        xs5 = [_gauss(RAGGED, 960 + i, role="worker") for i in range(5)]
        c5 = _gauss(RAGGED, 959, role="center")
        d_xs5, d_c5 = [to_device(x) for x in xs5], to_device(c5)
        px.easgd_round(table, [table.bufset(d) for d in d_xs5], table.bufset(d_c5), 0.0625)
        for x in xs5:
            oracle_mod.easgd_tensors(x, c5, 0.0625)
        assert_bits_equal(to_host(d_c5), c5, "round of 5 launch shape")
        for i in range(5):
            assert_bits_equal(to_host(d_xs5[i]), xs5[i], "round of 5 launch shape")
    finally:
        px.set_option(px.OPT_CHUNK_ELEMS, old[0])
        px.set_option(px.OPT_BLOCKS_PER_CU, old[1])


@pytest.mark.parametrize("policy", [-1, 0])
@pytest.mark.parametrize("offset", [0, 1])
def test_center_resident_option_gives_the_same_bits(px, oracle_mod, policy, offset):
    """Keeping the center in the memory-side cache changes how it is loaded and stored, never a result:
    single meetings and fused rounds of every specialised size, with the option on (each kernel's own cache
    policy and the plain one; the other policies are covered with the tuning build in test_gpu_policies.py)."""
    old = px.get_option(px.OPT_NONTEMPORAL)
    try:
        px.set_option(px.OPT_CENTER_RESIDENT, 1)
        px.set_option(px.OPT_NONTEMPORAL, policy)
        table = px.Table(RAGGED)
        for k in (1, 2, 3, 4, 5, 8, 9):
            xs = [_gauss(RAGGED, 970 + k, w, role="worker") for w in range(k)]
            c = _gauss(RAGGED, 971 + k, role="center")
            d_xs, d_c = [to_device(x, offset) for x in xs], to_device(c, offset)
            sets, sc = [table.bufset(x) for x in d_xs], table.bufset(d_c)
            px.easgd_round(table, sets, sc, 0.0625)
            px.easgd(table, sets[0], sc, 0.0625)
            for i in list(range(k)) + [0]:
                oracle_mod.easgd_tensors(xs[i], c, np.float32(0.0625))
            for i in range(k):
                assert_bits_equal(to_host(d_xs[i]), xs[i], f"k={k} x[{i}]")
            assert_bits_equal(to_host(d_c), c, f"k={k} center")
    finally:
        px.set_option(px.OPT_CENTER_RESIDENT, 0)
        px.set_option(px.OPT_NONTEMPORAL, old)


def test_options_of_one_table_override_the_process_wide_ones(px, oracle_mod):
    """An elastic server's table keeps its center cached and takes the plain cache policy, another table in the
    same process streams with the kernels' own policies; neither setting leaks, and results never depend on them."""
    t_server, t_other = px.Table(RAGGED), px.Table(RAGGED)
    t_server.set_option(px.OPT_CENTER_RESIDENT, 1)
    t_server.set_option(px.OPT_NONTEMPORAL, 0)
    assert t_server.get_option(px.OPT_CENTER_RESIDENT) == 1 and t_server.get_option(px.OPT_NONTEMPORAL) == 0
    assert t_other.get_option(px.OPT_CENTER_RESIDENT) == px.TABLE_OPTION_INHERIT
    assert px.get_option(px.OPT_CENTER_RESIDENT) == 0 and px.get_option(px.OPT_NONTEMPORAL) == -1
    assert t_server.view(3, 4).get_option(px.OPT_CENTER_RESIDENT) == 1           # a view follows its parent
    with pytest.raises(px.PxchgError):
        t_server.view(3, 4).set_option(px.OPT_CENTER_RESIDENT, 0)
    with pytest.raises(px.PxchgError) as e:
        t_server.set_option(px.OPT_NONTEMPORAL, 4)                               # the regular build holds -1 and 0
    assert e.value.status == 3
    for table in (t_server, t_other, t_server.view(0, len(RAGGED))):
        for k in (1, 2, 8):
            xs = [_gauss(RAGGED, 975 + k, w, role="worker") for w in range(k)]
            c = _gauss(RAGGED, 976 + k, role="center")
            root = t_server if table is not t_other else t_other
            d_xs, d_c = [to_device(x) for x in xs], to_device(c)
            sets, sc = [root.bufset(x) for x in d_xs], root.bufset(d_c)
            px.easgd_round(table, sets, sc, 0.0625)
            px.easgd(table, sets[0], sc, 0.0625)
            for i in list(range(k)) + [0]:
                oracle_mod.easgd_tensors(xs[i], c, np.float32(0.0625))
            for i in range(k):
                assert_bits_equal(to_host(d_xs[i]), xs[i], f"k={k} x[{i}]")
            assert_bits_equal(to_host(d_c), c, f"k={k} center")
    t_server.set_option(px.OPT_CENTER_RESIDENT, px.TABLE_OPTION_INHERIT)
    assert t_server.get_option(px.OPT_CENTER_RESIDENT) == px.TABLE_OPTION_INHERIT


# ------------------------------------------------------------------ argument errors on a live device

def test_argument_errors(px):
    import torch
    table = px.Table([100, 200])
    other = px.Table([100, 200])
    a = [torch.zeros(100, device="cuda"), torch.zeros(200, device="cuda")]
    h = [torch.zeros(100, device="cuda", dtype=torch.float16),
         torch.zeros(200, device="cuda", dtype=torch.float16)]
    sa, sh = table.bufset(a), table.bufset(h)
    so = other.bufset(a)
    with pytest.raises(px.PxchgError) as e:
        px.reduce_avg(table, [sa, so], sa)
    assert e.value.status == 2                         # set of another table
    with pytest.raises(px.PxchgError) as e:
        px.reduce_avg(table, [sa, sh], sa)
    assert e.value.status == 2                         # mixed element types
    with pytest.raises(px.PxchgError) as e:
        px.reduce_avg(table, [sa] * 65, sa)
    assert e.value.status == 3                         # k too large
    with pytest.raises(px.PxchgError) as e:
        px.sgd_momentum(table, sa, sa, sa, 0.1, 0.9)
    assert e.value.status == 1                         # aliasing operands
    with pytest.raises(px.PxchgError) as e:
        px.pack_fp16(table, [sh], [sa])
    assert e.value.status == 2
    with pytest.raises(px.PxchgError) as e:
        px.easgd(table, sa, sa, 0.1)
    assert e.value.status == 1
    # a tensor that does not fit its allocation is refused at set creation
    big = torch.zeros(16 << 20, device="cuda")          # 64 MiB, an allocation of its own
    too_long = px.Table([(16 << 20) + (4 << 20)])       # claims 16 MiB more than that
    with pytest.raises(px.PxchgError) as e:
        px.BufSet(too_long, [big.data_ptr()], px.F32)
    assert e.value.status == 6
    # misaligned for the element type
    with pytest.raises(px.PxchgError) as e:
        px.BufSet(table, [a[0].data_ptr() + 2, a[1].data_ptr()], px.F32)
    assert e.value.status == 1


# ------------------------------------------------------------------ diagnostics

def stats_order():
    """The parameters of the summation order that pxchg_buffer_stats is defined with, read from the header (they
    are part of the interface); the oracle takes them as arguments and shares no constant with the library."""
    import os
    import re
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "pxchg.h")).read()
    get = lambda name: int(re.search(rf"#define\s+{name}\s+(\d+)", text).group(1))  # noqa: E731
    return get("PXCHG_STATS_WAVES"), get("PXCHG_STATS_BLOCK_CHUNKS"), get("PXCHG_STATS_COMBINE_THREADS")


def oracle_stats(oracle_mod, tensors, chunk=512):
    return oracle_mod.stats_ordered_tensors(tensors, chunk, *stats_order())


@pytest.mark.parametrize("dt", [np.float32, np.float16])
@pytest.mark.parametrize("offset", [0, 1, 3])
def test_buffer_stats(px, oracle_mod, dt, offset):
    """Count, maximum and the tree-ordered sum of squares equal the oracle bit for bit: ragged tensors, operands
    off 16-byte alignment (the order is a matter of element indices, not of addresses), elements that are not
    finite; and the same bits on every call."""
    import torch
    table = px.Table(RAGGED)
    a = [t.astype(dt) for t in _gauss(RAGGED, 970)]
    a[7][[3, 500, 19_999]] = [np.inf, np.nan, -np.inf]
    a[11][70_000] = -7.25
    a[0][0] = np.nan
    d_a = to_device(a, offset)
    out = torch.full((4,), -1, dtype=torch.int64, device="cuda")     # garbage in: the call overwrites it
    want = oracle_stats(oracle_mod, a)
    assert want[:2] == (4, 7.25) and want[:2] == oracle_mod.stats_tensors(a)[:2]
    assert abs(want[2] - oracle_mod.stats_tensors(a)[2]) <= 1e-13 * want[2]
    for _ in range(3):
        px.buffer_stats(table, table.bufset(d_a), out)
        torch.cuda.synchronize()
        assert px.read_stats(out) == want
        out[:3].fill_(-1)
    assert int(out[3].item()) == -1                                  # nothing past the 24 bytes was touched


def test_buffer_stats_order_decides_roundings_as_defined(px, oracle_mod):
    """Inputs whose sum of squares depends on the order of addition (one element with a square of 2^54 among
    elements with a square of 1: a lone 1 added to 2^54 is lost, four of them added up first are kept), placed so
    that lane, wavefront, block and final-combine ownership each decide the result.  The library must land on
    the oracle's bits, which differ from the index-order sum here."""
    import torch
    waves, block, _ = stats_order()
    n = 512 * block * 3 + 700                                        # three blocks and a ragged fourth
    rng = np.random.default_rng(4)
    for trial in range(4):
        a = np.zeros(n, np.float32)
        a[rng.integers(0, n, 3000)] = 1.0
        a[rng.integers(0, n, 3)] = 2.0 ** 27
        a[[0, 512 * waves, 512 * block, n - 1]] = [2.0 ** 27, 1.0, 1.0, 1.0]
        table = px.Table([n])
        out = torch.zeros(3, dtype=torch.int64, device="cuda")
        px.buffer_stats(table, table.bufset(to_device([a])), out)
        torch.cuda.synchronize()
        want = oracle_stats(oracle_mod, [a])
        assert px.read_stats(out) == want
        assert want[2] != oracle_mod.stats(a)[2]                     # the order matters on this input


@pytest.mark.parametrize("chunk", [1024, 8192])
def test_buffer_stats_other_chunk_sizes(px, oracle_mod, chunk):
    import torch
    old = px.get_option(px.OPT_CHUNK_ELEMS)
    try:
        px.set_option(px.OPT_CHUNK_ELEMS, chunk)
        table = px.Table(RAGGED)
        for dt in (np.float32, np.float16):
            a = [t.astype(dt) for t in _gauss(RAGGED, 973)]
            out = torch.zeros(3, dtype=torch.int64, device="cuda")
            px.buffer_stats(table, table.bufset(to_device(a)), out)
            torch.cuda.synchronize()
            assert px.read_stats(out) == oracle_stats(oracle_mod, a, chunk)
    finally:
        px.set_option(px.OPT_CHUNK_ELEMS, old)


def test_buffer_stats_sees_overflow_of_the_pack(px, oracle_mod):
    import torch
    counts = [5000, 8192 * 2 + 1]
    table = px.Table(counts)
    g = _gauss(counts, 971)
    g[1][[10, 9000]] = [7.0e4, -1.0e5]                               # beyond the binary16 range
    d_g = to_device(g)
    d_h = empty_like_device(counts, np.float16)
    s_g, s_h = table.bufset(d_g), table.bufset(d_h)
    px.pack_fp16(table, [s_g], [s_h])
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    px.buffer_stats(table, s_g, out)
    torch.cuda.synchronize()
    assert px.read_stats(out)[0] == 0
    px.buffer_stats(table, s_h, out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == oracle_stats(oracle_mod, oracle_mod.pack_fp16_tensors(g))
    assert px.read_stats(out)[0] == 2


@pytest.mark.parametrize("dt", [np.float16, np.float32])
def test_buffer_stats_full_size(px, oracle_mod, dt):
    """AlexNet-shaped buffer, every element: the same bits as the oracle's ordered sum, on five calls in a row."""
    import torch
    counts = wl.alexnet_counts()
    table = px.Table(counts)
    a = [t.astype(dt) for t in wl.gaussian_tensors(counts, 0.01, 972, "grad")]
    d_a = to_device(a)
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    want = oracle_stats(oracle_mod, a)
    for _ in range(5):
        px.buffer_stats(table, table.bufset(d_a), out)
        torch.cuda.synchronize()
        assert px.read_stats(out) == want
    # and that sum is a good one: within a few units in the last place of numpy's pairwise binary64 sum
    exact = float(sum(np.sum(t.astype(np.float64) ** 2) for t in a))
    assert want[0] == 0 and abs(want[2] - exact) <= 1e-14 * exact
    with pytest.raises(px.PxchgError):
        px.buffer_stats(table, table.bufset(d_a), out.data_ptr() + 4)   # misaligned output


# ------------------------------------------------------------------ layer by layer, on two streams

def test_per_layer_exchange_on_two_streams_equals_whole_set(px, oracle_mod):
    """The exchange of one layer does not depend on the others, so layers can be exchanged as their
    gradients become ready, on different streams (the overlap the paper names as future work).  One
    table per layer, alternating streams; results equal the oracle on the whole set."""
    import torch
    counts = [34_848, 96, 307_200, 256, 100_003, 1000]
    k = 4
    grads = [_gauss(counts, 980, w) for w in range(k)]
    w = _gauss(counts, 981, role="param")
    v = wl.zeros_tensors(counts)
    d_g = [to_device(g) for g in grads]
    d_w, d_v = to_device(w), to_device(v)
    d_avg = empty_like_device(counts, np.float32)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    keep = []
    for layer in reversed(range(len(counts) // 2)):          # last layer's gradients are ready first
        sl = slice(2 * layer, 2 * layer + 2)                  # weight and bias of this layer
        table = px.Table(counts[sl])
        sets = [table.bufset(d_g[i][sl]) for i in range(k)]
        s_avg, s_w, s_v = table.bufset(d_avg[sl]), table.bufset(d_w[sl]), table.bufset(d_v[sl])
        st = streams[layer % 2]
        px.reduce_avg(table, sets, s_avg, px.AVG, stream=st)
        px.sgd_momentum(table, s_avg, s_w, s_v, 0.01, 0.9, 5e-4, stream=st)
        keep.append((table, sets, s_avg, s_w, s_v))
    for st in streams:
        st.synchronize()
    avg = oracle_mod.reduce_avg_tensors(grads)
    oracle_mod.sgd_momentum_tensors(avg, w, v, 0.01, 0.9, 5e-4)
    assert_bits_equal(to_host(d_w), w, "w")
    assert_bits_equal(to_host(d_v), v, "v")


def test_views_exchange_layer_by_layer_with_the_parents_sets(px, oracle_mod):
    """pxchg_table_view: every call restricted to a run of tensors, with the parent's buffer sets and
    multipliers.  Layer by layer on two streams (staged for some layers, fused for others), then the elastic
    round, the conversions and the diagnostics through views; everything equals the whole-set oracle."""
    import torch
    counts = [34_848, 96, 0, 20_001, 3, 8192 * 2 + 5, 1000, 513, 70_000, 7]
    k = 3
    table = px.Table(counts)
    lr_mult = [1.0, 2.0, 1.0, 1.0, 2.0, 1.0, 2.0, 0.5, 1.0, 2.0]
    wd_mult = [1.0, 0.0, 1.0, 1.0, 0.0, 1.0, 0.0, 1.0, 1.0, 0.0]
    table.set_multipliers(lr_mult, wd_mult)
    grads = [_gauss(counts, 1100, w) for w in range(k)]
    w = _gauss(counts, 1101, role="param")
    v = _gauss(counts, 1102, sigma=1e-3, role="velocity")
    xs = [_gauss(counts, 1103, i, role="worker") for i in range(k)]
    c = _gauss(counts, 1104, role="center")
    d_g = [to_device(g) for g in grads]
    d_h = [empty_like_device(counts, np.float16) for _ in range(k)]
    d_avg = empty_like_device(counts, np.float16)
    d_w, d_v = to_device(w), to_device(v)
    d_xs, d_c = [to_device(x) for x in xs], to_device(c)
    s_g, s_h = [table.bufset(t) for t in d_g], [table.bufset(t) for t in d_h]
    s_avg, s_w, s_v = table.bufset(d_avg), table.bufset(d_w), table.bufset(d_v)
    s_xs, s_c = [table.bufset(t) for t in d_xs], table.bufset(d_c)
    layers = [(8, 2), (6, 2), (3, 3), (2, 1), (0, 2)]            # (first tensor, tensors), last layer first
    assert sorted(t for f, m in layers for t in range(f, f + m)) == list(range(len(counts)))
    views = [table.view(f, m) for f, m in layers]
    assert [vw.total for vw in views] == [sum(counts[f:f + m]) for f, m in layers]
    assert sum(vw.n_chunks for vw in views) == table.n_chunks
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for li, vw in enumerate(views):
        st = streams[li % 2]
        px.pack_fp16(vw, s_g, s_h, stream=st)
        if li % 2 == 0:
            px.reduce_avg(vw, s_h, s_avg, stream=st)
            px.sgd_momentum(vw, s_avg, s_w, s_v, 0.01, 0.9, 5e-4, stream=st)
        else:
            px.reduce_avg_sgd_momentum(vw, s_h, s_w, s_v, 0.01, 0.9, 5e-4, px.AVG, px.F16, stream=st)
        px.easgd_round(vw, s_xs, s_c, 0.125, stream=st)
    for st in streams:
        st.synchronize()
    packed = [oracle_mod.pack_fp16_tensors(g) for g in grads]
    avg = oracle_mod.reduce_avg_tensors(packed, np.float16)
    for t in range(len(counts)):
        oracle_mod.sgd_momentum(avg[t], w[t], v[t], float(np.float32(0.01) * np.float32(lr_mult[t])), 0.9,
                                float(np.float32(5e-4) * np.float32(wd_mult[t])))
    for i in range(k):
        oracle_mod.easgd_tensors(xs[i], c, 0.125)
    for i in range(k):
        assert_bits_equal(to_host(d_h[i]), packed[i], f"packed[{i}]")
        assert_bits_equal(to_host(d_xs[i]), xs[i], f"x[{i}]")
    assert_bits_equal(to_host(d_w), w, "w")
    assert_bits_equal(to_host(d_v), v, "v")
    assert_bits_equal(to_host(d_c), c, "center")
    # the staged layers wrote their part of the mean, the fused ones left theirs alone
    got_avg = to_host(d_avg)
    for li, (f, m) in enumerate(layers):
        if li % 2 == 0:
            assert_bits_equal(got_avg[f:f + m], avg[f:f + m], f"mean of layer {li}")
    # diagnostics and widening through a view see only its tensors
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    px.buffer_stats(views[0], s_w, out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == oracle_stats(oracle_mod, w[8:10])     # the view's own chunk list defines the order
    d_back = empty_like_device(counts, np.float32, fill=7.0)
    px.unpack_fp16(views[2], [s_h[0]], [table.bufset(d_back)])
    back = to_host(d_back)
    assert_bits_equal(back[3:6], oracle_mod.unpack_fp16_tensors(packed[0][3:6]), "unpack through a view")
    assert all(np.all(b == 7.0) for t, b in enumerate(back) if not 3 <= t < 6)


def test_grouped_views_cover_the_set_and_exchange_like_the_whole_set(px, oracle_mod):
    """Table.bucketed_views: runs of consecutive tensors of at least a given size, formed from the last tensor
    backwards (the order in which back-propagation hands gradients over), small layers sharing a group.  The
    AlexNet shapes give three groups; a producer stream packs each group and the exchange stream reduces and
    updates it as soon as its event fires; the result equals the oracle on the whole set."""
    import torch
    counts = wl.alexnet_counts()
    table = px.Table(counts)
    groups = table.bucketed_views(8_000_000)
    assert [(g.counts[0], len(g.counts)) for g in groups] == [(16_777_216, 4), (37_748_736, 2), (34_848, 10)]
    assert sum(g.total for g in groups) == sum(counts) and sum(g.n_chunks for g in groups) == table.n_chunks
    assert [g.total for g in table.bucketed_views(10 ** 9)] == [sum(counts)]            # one group if nothing is big enough
    assert len(table.bucketed_views(1)) == len(counts)                                  # every tensor its own group
    assert [len(g.counts) for g in table.bucketed_views(8_000_000, reverse=False)] == [11, 2, 3]
    k = 3
    grads = [_gauss(counts, 1300, w) for w in range(k)]
    w, v = _gauss(counts, 1301, role="param"), wl.zeros_tensors(counts)
    d_g = [to_device(g) for g in grads]
    d_h = [empty_like_device(counts, np.float16) for _ in range(k)]
    d_avg, d_w, d_v = empty_like_device(counts, np.float16), to_device(w), to_device(v)
    s_g, s_h = [table.bufset(t) for t in d_g], [table.bufset(t) for t in d_h]
    s_avg, s_w, s_v = table.bufset(d_avg), table.bufset(d_w), table.bufset(d_v)
    producer, exchange = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for gi, grp in enumerate(groups):
        px.pack_fp16(grp, s_g, s_h, stream=producer)
        ready = torch.cuda.Event()
        ready.record(producer)
        exchange.wait_event(ready)
        if gi == 1:
            px.reduce_avg_sgd_momentum(grp, s_h, s_w, s_v, 0.01, 0.9, 5e-4, px.AVG, px.F16, stream=exchange)
        else:
            px.reduce_avg(grp, s_h, s_avg, stream=exchange)
            px.sgd_momentum(grp, s_avg, s_w, s_v, 0.01, 0.9, 5e-4, stream=exchange)
    exchange.synchronize()
    packed = [oracle_mod.pack_fp16_tensors(g) for g in grads]
    avg = oracle_mod.reduce_avg_tensors(packed, np.float16)
    oracle_mod.sgd_momentum_tensors(avg, w, v, 0.01, 0.9, 5e-4)
    assert_bits_equal(to_host(d_w), w, "w")
    assert_bits_equal(to_host(d_v), v, "v")


def test_view_argument_errors(px):
    import torch
    table = px.Table([100, 200, 300])
    other = px.Table([100, 200, 300])
    a = [torch.zeros(c, device="cuda") for c in (100, 200, 300)]
    sa, so = table.bufset(a), other.bufset([t.clone() for t in a])
    view = table.view(1, 2)
    assert (view.total, view.n_tensors, view.n_chunks) == (500, 2, 2)
    for first, m in ((-1, 1), (0, 0), (0, 4), (3, 1), (2, 2)):
        with pytest.raises(px.PxchgError) as e:
            table.view(first, m)
        assert e.value.status == 1
    with pytest.raises(px.PxchgError) as e:
        view.view(0, 1)                                   # no views of views
    assert e.value.status == 1
    with pytest.raises(px.PxchgError) as e:
        view.bufset(a[1:])                                # sets belong to the parent
    assert e.value.status == 1
    with pytest.raises(px.PxchgError) as e:
        view.set_multipliers([1.0, 1.0], None)
    assert e.value.status == 1
    with pytest.raises(px.PxchgError) as e:
        px.easgd(view, sa, so, 0.1)                       # a set of another table
    assert e.value.status == 2
    empty = px.Table([0, 5, 0]).view(0, 1)
    assert empty.n_chunks == 0 and empty.total == 0


# ------------------------------------------------------------------ degenerate and maximum sizes

def test_table_of_empty_tensors_is_a_no_op(px):
    import torch
    table = px.Table([0, 0, 0])
    assert table.total == 0 and table.n_chunks == 0
    s32 = px.BufSet(table, [0, 0, 0], px.F32)
    s32b = px.BufSet(table, [0, 0, 0], px.F32)
    s32c = px.BufSet(table, [0, 0, 0], px.F32)
    s16 = px.BufSet(table, [0, 0, 0], px.F16)
    px.pack_fp16(table, [s32], [s16])
    px.unpack_fp16(table, [s16], [s32])
    px.reduce_avg(table, [s32, s32b], s32c)
    px.sgd_momentum(table, s16, s32, s32b, 0.1, 0.9, 0.0)
    px.easgd(table, s32, s32b, 0.5)
    px.easgd_round(table, [s32, s32b], s32c, 0.5)
    px.reduce_avg_sgd_momentum(table, [s16], s32, s32b, 0.1, 0.9)
    out = torch.full((3,), 5, dtype=torch.int64, device="cuda")
    px.buffer_stats(table, s16, out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == (0, 0.0, 0.0)


def test_one_tensor_longer_than_2_to_the_31_elements(px, oracle_mod):
    """64-bit element offsets: a single binary16 tensor of 2^31 + 1,029 elements is widened on the GPU and
    compared with the oracle on windows at the start, around the 2^31 boundary, at the end and in between."""
    import torch
    n = (1 << 31) + 1029
    rng = np.random.default_rng(99)
    block = rng.integers(0, 1 << 16, 1 << 22, dtype=np.uint16)          # all kinds of halves, NaN included
    table = px.Table([n])
    d_h = torch.empty(n, dtype=torch.float16, device="cuda")
    d_blk = torch.from_numpy(block.view(np.float16)).cuda()
    reps = n // block.size
    d_h[:reps * block.size].view(reps, block.size).copy_(d_blk.expand(reps, block.size))
    d_h[reps * block.size:].copy_(d_blk[:n - reps * block.size])
    d_f = torch.empty(n, dtype=torch.float32, device="cuda")
    px.unpack_fp16(table, [table.bufset([d_h])], [table.bufset([d_f])])
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    px.buffer_stats(table, table.bufset([d_h]), out)
    torch.cuda.synchronize()
    windows = [0, 12_345_678, (1 << 31) - 2048, (1 << 31) - 5, n - 4099, n - 1029]
    for s in windows:
        e = min(n, s + 4099)
        idx = np.arange(s, e) % block.size
        want = oracle_mod.unpack_fp16(np.ascontiguousarray(block[idx]).view(np.float16))
        got = d_f[s:e].cpu().numpy()
        assert_bits_equal([got], [want], f"window at {s}", nan_as_class=True)
    # the count of non-finite halves over all n elements follows from the block
    exp = (block >> 10) & 0x1F
    per_block = int(np.count_nonzero(exp == 0x1F))
    tail = int(np.count_nonzero(exp[:n - reps * block.size] == 0x1F))
    assert px.read_stats(out)[0] == reps * per_block + tail
    del d_f, d_h
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ a whole step captured in a HIP graph

def test_exchange_step_replayed_from_a_hip_graph(px, oracle_mod):
    """The calls allocate nothing, copy nothing from the host and record no memset, so a step can be captured
    once and replayed.  Three replays with fresh gradients written between them (eager work and
    synchronisations in between), each checked against the oracle."""
    import torch
    counts = [34_848, 96, 20_001, 3, 8192 * 2 + 5, 1000]
    k = 4
    table = px.Table(counts)
    w = _gauss(counts, 990, role="param")
    v = wl.zeros_tensors(counts)
    xs = [_gauss(counts, 991, i, role="worker") for i in range(k)]
    c = _gauss(counts, 992, role="center")
    d_g = [to_device(_gauss(counts, 993, i)) for i in range(k)]
    d_h = [empty_like_device(counts, np.float16) for _ in range(k)]
    d_avg = empty_like_device(counts, np.float16)
    d_w, d_v = to_device(w), to_device(v)
    d_xs, d_c = [to_device(x) for x in xs], to_device(c)
    d_stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    s_g, s_h = [table.bufset(t) for t in d_g], [table.bufset(t) for t in d_h]
    s_avg, s_w, s_v = table.bufset(d_avg), table.bufset(d_w), table.bufset(d_v)
    s_xs, s_c = [table.bufset(t) for t in d_xs], table.bufset(d_c)

    def step():
        px.pack_fp16(table, s_g, s_h)
        px.reduce_avg(table, s_h, s_avg)
        px.buffer_stats(table, s_avg, d_stats)
        px.sgd_momentum(table, s_avg, s_w, s_v, 0.01, 0.9, 5e-4)
        for i in range(k):
            px.easgd(table, s_xs[i], s_c, 0.125)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        snapshot = [t.clone() for t in d_w + d_v + d_c] + [t.clone() for x in d_xs for t in x]
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capture does not execute: state is unchanged
    for a, b in zip(d_w + d_v + d_c + [t for x in d_xs for t in x], snapshot):
        assert torch.equal(a, b)
    for r in range(3):
        grads = [_gauss(counts, 994 + r, i) for i in range(k)]
        for i in range(k):
            for dst, src in zip(d_g[i], grads[i]):
                dst.copy_(torch.from_numpy(src))                 # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        packed = [oracle_mod.pack_fp16_tensors(g) for g in grads]
        avg = oracle_mod.reduce_avg_tensors(packed, np.float16)
        oracle_mod.sgd_momentum_tensors(avg, w, v, 0.01, 0.9, 5e-4)
        for i in range(k):
            oracle_mod.easgd_tensors(xs[i], c, 0.125)
        assert_bits_equal(to_host(d_avg), avg, f"replay {r} average")
        assert_bits_equal(to_host(d_w), w, f"replay {r} w")
        assert_bits_equal(to_host(d_v), v, f"replay {r} v")
        assert_bits_equal(to_host(d_c), c, f"replay {r} center")
        assert_bits_equal(to_host(d_xs[k - 1]), xs[k - 1], f"replay {r} worker")
        assert px.read_stats(d_stats) == oracle_stats(oracle_mod, avg)


def test_destroying_unrelated_objects_does_not_break_a_capture(px, oracle_mod):
    """A garbage collector may drop an old table or buffer set at any moment, also while a stream is being
    captured into a graph.  Destruction waits for the device and frees memory, which a capture in progress would
    answer by invalidating itself; the binding puts such a handle aside and destroys it after the capture."""
    import torch
    counts = [5000, 77]
    table = px.Table(counts)
    x, c = _gauss(counts, 1200, role="worker"), _gauss(counts, 1201, role="center")
    d_x, d_c = to_device(x), to_device(c)
    sx, sc = table.bufset(d_x), table.bufset(d_c)
    old_table = px.Table([123, 4567])
    old_set = old_table.bufset([torch.zeros(123, device="cuda"), torch.zeros(4567, device="cuda")])
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            px.easgd(table, sx, sc, 0.25)
            old_set.close()                     # what a collector would do, in the middle of the capture
            old_table.close()
            put_aside = len(px.binding._deferred)
            px.easgd(table, sx, sc, 0.25)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert put_aside >= 2                       # both were put aside during the capture ...
    px.flush_deferred()
    assert not px.binding._deferred             # ... and are destroyed now
    for r in range(2):
        graph.replay()
        torch.cuda.synchronize()
        for _ in range(2):
            oracle_mod.easgd_tensors(x, c, 0.25)
        assert_bits_equal(to_host(d_x), x, f"replay {r} x")
        assert_bits_equal(to_host(d_c), c, f"replay {r} center")


# ------------------------------------------------------------------ per-tensor multipliers

@pytest.mark.parametrize("fused", [False, True])
def test_per_tensor_learning_rate_and_decay_multipliers(px, oracle_mod, fused):
    """Biases with twice the learning rate and no weight decay, one frozen tensor: tensor t is updated with
    lr * lr_mult[t] and wd * wd_mult[t] (products rounded to binary32), as a per-tensor oracle call."""
    counts = [34_848, 96, 20_001, 3, 8192 * 2 + 5, 1000]
    lr_mult = [1.0, 2.0, 1.0, 2.0, 0.0, 0.3]
    wd_mult = [1.0, 0.0, 1.0, 0.0, 1.0, 2.5]
    k, lr, mu, wd = 3, 0.01, 0.9, 5e-4
    table = px.Table(counts)
    table.set_multipliers(lr_mult, wd_mult)
    grads = [_gauss(counts, 1000, i) for i in range(k)]
    w, v = _gauss(counts, 1001, role="param"), _gauss(counts, 1002, sigma=1e-3, role="velocity")
    w_before = [a.copy() for a in w]
    d_w, d_v = to_device(w), to_device(v)
    s_g = [table.bufset(to_device(g)) for g in grads]
    s_w, s_v = table.bufset(d_w), table.bufset(d_v)
    if fused:
        px.reduce_avg_sgd_momentum(table, s_g, s_w, s_v, lr, mu, wd, px.AVG, px.F32)
    else:
        d_avg = empty_like_device(counts, np.float32)
        s_avg = table.bufset(d_avg)
        px.reduce_avg(table, s_g, s_avg)
        px.sgd_momentum(table, s_avg, s_w, s_v, lr, mu, wd)
    avg = oracle_mod.reduce_avg_tensors(grads)
    for t in range(len(counts)):
        lr_t = np.float32(lr) * np.float32(lr_mult[t])
        wd_t = np.float32(wd) * np.float32(wd_mult[t])
        oracle_mod.sgd_momentum(avg[t], w[t], v[t], lr_t, mu, wd_t)
    assert_bits_equal(to_host(d_w), w, "w")
    assert_bits_equal(to_host(d_v), v, "v")
    assert np.any(w[0] != w_before[0])
    # removing the multipliers restores the plain behaviour
    table.set_multipliers(None, None)
    w2, v2 = _gauss(counts, 1001, role="param"), _gauss(counts, 1002, sigma=1e-3, role="velocity")
    d_w2, d_v2 = to_device(w2), to_device(v2)
    d_avg = to_device(avg)
    px.sgd_momentum(table, table.bufset(d_avg), table.bufset(d_w2), table.bufset(d_v2), lr, mu, wd)
    oracle_mod.sgd_momentum_tensors(avg, w2, v2, lr, mu, wd)
    assert_bits_equal(to_host(d_w2), w2, "w without multipliers")
