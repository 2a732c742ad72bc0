"""Cache policies never change a result.  Every kernel exists with six load/store policies in the tuning build of
the library (tests/_build/libpxchg_allpolicies.so, made by __graft_entry__.build() with -DPXCHG_ALL_POLICIES);
two of them store through hand-written instructions that need wait states before their data registers may be
overwritten.  This file runs every call under every policy on a ragged multi-tensor set (a few hundred thousand
elements, one tensor of 70,001) and compares every element with the oracle, bit for bit: above all the kernel
shapes that issue the most 16-byte stores in a row per lane (the fused reduce+update with binary16 contributions
and two workers: four; the elastic round of two: three; the float32 reduce of up to three workers and the
widening unpack: two), also with larger chunks, where a lane repeats its vector step several times."""
import os

import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_bits_equal, empty_like_device, to_device, to_host

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TUNING_LIB = os.path.join(ROOT, "tests", "_build", "libpxchg_allpolicies.so")
COUNTS = [1, 3, 63, 64, 65, 0, 8 * 1000 + 1, 20_000, 2 * 8192 + 5, 8192, 8191, 70_001, 131_072, 4 * 8192 + 3]
POLICIES = [0, 1, 2, 3, 4, 5]


@pytest.fixture(scope="module")
def px():
    """The package, with the tuning build as the library that new tables are made with."""
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1605_08325_amd as px
    if not os.path.exists(TUNING_LIB):
        pytest.skip("tests/_build/libpxchg_allpolicies.so is not built: run __graft_entry__.build() first")
    lib = px.open_library(TUNING_LIB)
    with px.using(lib):
        assert px.get_option(px.OPT_ALL_POLICIES_BUILT) == 1
        yield px
        px.set_option(px.OPT_NONTEMPORAL, -1)
        px.set_option(px.OPT_CENTER_RESIDENT, 0)
        px.set_option(px.OPT_CHUNK_ELEMS, 512)


def _gauss(seed, worker=0, sigma=0.01, role="grad"):
    return [a.copy() for a in wl.gaussian_tensors(COUNTS, sigma, seed, role, worker)]


def test_the_regular_build_refuses_the_tuning_policies():
    import paper_1605_08325_amd as regular
    with regular.using(regular.open_library(regular.library_path())):      # whatever library the tests around it use
        assert regular.get_option(regular.OPT_ALL_POLICIES_BUILT) == 0
        for policy in (1, 2, 3, 4, 5):
            with pytest.raises(regular.PxchgError) as e:
                regular.set_option(regular.OPT_NONTEMPORAL, policy)
            assert e.value.status == 3
        regular.set_option(regular.OPT_NONTEMPORAL, 0)
        regular.set_option(regular.OPT_NONTEMPORAL, -1)


@pytest.mark.parametrize("chunk", [512, 2048, 8192])
@pytest.mark.parametrize("policy", POLICIES)
def test_conversions_and_reduce(px, oracle_mod, policy, chunk):
    px.set_option(px.OPT_NONTEMPORAL, policy)
    px.set_option(px.OPT_CHUNK_ELEMS, chunk)
    table = px.Table(COUNTS)
    k = 3
    g = [_gauss(962, w) for w in range(k)]
    s_g = [table.bufset(to_device(t)) for t in g]
    d_h = [empty_like_device(COUNTS, np.float16) for _ in range(k)]
    s_h = [table.bufset(t) for t in d_h]
    px.pack_fp16(table, s_g, s_h)
    packed = [oracle_mod.pack_fp16_tensors(t) for t in g]
    for w in range(k):
        assert_bits_equal(to_host(d_h[w]), packed[w], "pack")
    d_back = [empty_like_device(COUNTS, np.float32) for _ in range(k)]
    px.unpack_fp16(table, s_h, [table.bufset(t) for t in d_back])
    for w in range(k):
        assert_bits_equal(to_host(d_back[w]), oracle_mod.unpack_fp16_tensors(packed[w]), "unpack")
    # every combination of element types; 1..3 workers take the widest lanes, 8 and 9 the other kernel shapes
    for kk in (1, 2, 3, 8, 9):
        g32 = [_gauss(963, w) for w in range(kk)]
        g16 = [oracle_mod.pack_fp16_tensors(t) for t in g32]
        sets = {np.float32: [table.bufset(to_device(t)) for t in g32],
                np.float16: [table.bufset(to_device(t)) for t in g16]}
        host = {np.float32: g32, np.float16: g16}
        for in_dt in (np.float32, np.float16):
            for out_dt in (np.float32, np.float16):
                d_out = empty_like_device(COUNTS, out_dt)
                px.reduce_avg(table, sets[in_dt], table.bufset(d_out))
                assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(host[in_dt], out_dt),
                                  f"reduce k={kk} {in_dt.__name__}->{out_dt.__name__}")
    if chunk == 512:
        _reduce_on_a_table_of_large_tensors(px, oracle_mod)


# One tensor of more than 512 chunks: the launch then takes the reduce that reads its pointers with scalar loads
# (the tables above, of many small tensors, take the one that fetches them lane-parallel) and the fused
# reduce+update with an idle wavefront.
LARGE = [300_001]
HUGE = [2_100_003]


def _reduce_on_a_table_of_large_tensors(px, oracle_mod):
    table = px.Table(LARGE)
    assert table.n_chunks > 512 * len(LARGE)
    for kk in (1, 3, 8):
        g32 = [[a.copy() for a in wl.gaussian_tensors(LARGE, 0.01, 970, "grad", w)] for w in range(kk)]
        g16 = [oracle_mod.pack_fp16_tensors(t) for t in g32]
        sets = {np.float32: [table.bufset(to_device(t)) for t in g32],
                np.float16: [table.bufset(to_device(t)) for t in g16]}
        host = {np.float32: g32, np.float16: g16}
        for in_dt in (np.float32, np.float16):
            for out_dt in (np.float32, np.float16):
                d_out = empty_like_device(LARGE, out_dt)
                px.reduce_avg(table, sets[in_dt], table.bufset(d_out))
                assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(host[in_dt], out_dt),
                                  f"large tensor, reduce k={kk} {in_dt.__name__}->{out_dt.__name__}")
    # from 4096 chunks per tensor on, the binary16 reduce of four or more workers runs with idle wavefronts
    table = px.Table(HUGE)
    assert table.n_chunks >= 4096 * len(HUGE)
    for kk in (4, 8):
        g16 = [oracle_mod.pack_fp16_tensors([a.copy() for a in wl.gaussian_tensors(HUGE, 0.01, 975, "grad", w)])
               for w in range(kk)]
        d_out = empty_like_device(HUGE, np.float16)
        px.reduce_avg(table, [table.bufset(to_device(t)) for t in g16], table.bufset(d_out))
        assert_bits_equal(to_host(d_out), oracle_mod.reduce_avg_tensors(g16, np.float16), f"huge tensor, reduce k={kk}")


@pytest.mark.parametrize("chunk", [512, 2048, 8192])
@pytest.mark.parametrize("policy", POLICIES)
def test_updates(px, oracle_mod, policy, chunk):
    px.set_option(px.OPT_NONTEMPORAL, policy)
    px.set_option(px.OPT_CHUNK_ELEMS, chunk)
    table = px.Table(COUNTS)
    for g_dt in (np.float32, np.float16):
        grad = [a.astype(g_dt) for a in _gauss(964)]
        w_, v_ = _gauss(965, role="param"), _gauss(966, sigma=1e-3, role="velocity")
        d_w, d_v = to_device(w_), to_device(v_)
        px.sgd_momentum(table, table.bufset(to_device(grad)), table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4)
        oracle_mod.sgd_momentum_tensors(grad, w_, v_, 0.01, 0.9, 5e-4)
        assert_bits_equal(to_host(d_w), w_, "w")
        assert_bits_equal(to_host(d_v), v_, "v")
    # fused reduce+update: binary16 and float32 contributions, both wire types
    for k in (1, 2, 3, 8, 9):
        g32 = [_gauss(967 + k, w) for w in range(k)]
        for in_dt in (np.float16, np.float32):
            contrib = [[a.astype(in_dt) for a in t] for t in g32]
            sets = [table.bufset(to_device(t)) for t in contrib]
            for wire_np, wire_px in ((np.float16, px.F16), (np.float32, px.F32)):
                w_, v_ = _gauss(968, role="param"), _gauss(969, sigma=1e-3, role="velocity")
                d_w, d_v = to_device(w_), to_device(v_)
                px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4,
                                           px.AVG, wire_px)
                avg = oracle_mod.reduce_avg_tensors(contrib, wire_np)
                oracle_mod.sgd_momentum_tensors(avg, w_, v_, 0.01, 0.9, 5e-4)
                assert_bits_equal(to_host(d_w), w_, f"fused k={k} {in_dt.__name__} wire {wire_np.__name__} w")
                assert_bits_equal(to_host(d_v), v_, f"fused k={k} {in_dt.__name__} wire {wire_np.__name__} v")
    if chunk == 512:  # the fused kernel's build with an idle wavefront (tables of large tensors)
        table = px.Table(LARGE)
        for k in (3, 8):
            g32 = [[a.copy() for a in wl.gaussian_tensors(LARGE, 0.01, 980 + k, "grad", w)] for w in range(k)]
            for in_dt in (np.float16, np.float32):
                contrib = [[a.astype(in_dt) for a in t] for t in g32]
                sets = [table.bufset(to_device(t)) for t in contrib]
                w_ = [a.copy() for a in wl.gaussian_tensors(LARGE, 0.01, 981, "param")]
                v_ = [a.copy() for a in wl.gaussian_tensors(LARGE, 1e-3, 982, "velocity")]
                d_w, d_v = to_device(w_), to_device(v_)
                px.reduce_avg_sgd_momentum(table, sets, table.bufset(d_w), table.bufset(d_v), 0.01, 0.9, 5e-4,
                                           px.AVG, px.F16)
                avg = oracle_mod.reduce_avg_tensors(contrib, np.float16)
                oracle_mod.sgd_momentum_tensors(avg, w_, v_, 0.01, 0.9, 5e-4)
                assert_bits_equal(to_host(d_w), w_, f"large tensor, fused k={k} {in_dt.__name__} w")
                assert_bits_equal(to_host(d_v), v_, f"large tensor, fused k={k} {in_dt.__name__} v")


@pytest.mark.parametrize("center_resident", [0, 1])
@pytest.mark.parametrize("chunk", [512, 2048])
@pytest.mark.parametrize("policy", POLICIES)
def test_elastic(px, oracle_mod, policy, chunk, center_resident):
    px.set_option(px.OPT_NONTEMPORAL, policy)
    px.set_option(px.OPT_CHUNK_ELEMS, chunk)
    px.set_option(px.OPT_CENTER_RESIDENT, center_resident)
    table = px.Table(COUNTS)
    for k in (1, 2, 3, 4, 5, 8, 9):
        xs = [_gauss(970 + k, w, role="worker") for w in range(k)]
        c = _gauss(971 + k, role="center")
        d_xs, d_c = [to_device(x) for x in xs], to_device(c)
        sets, sc = [table.bufset(x) for x in d_xs], table.bufset(d_c)
        px.easgd_round(table, sets, sc, 0.0625)
        px.easgd(table, sets[0], sc, 0.0625)
        for i in list(range(k)) + [0]:
            oracle_mod.easgd_tensors(xs[i], c, np.float32(0.0625))
        for i in range(k):
            assert_bits_equal(to_host(d_xs[i]), xs[i], f"k={k} x[{i}]")
        assert_bits_equal(to_host(d_c), c, f"k={k} center")


def test_policy_of_one_table_only(px, oracle_mod):
    """pxchg_table_set_option with the tuning build: two tables in one process under different policies."""
    px.set_option(px.OPT_NONTEMPORAL, -1)           # whatever the tests before left behind
    tables = {p: px.Table(COUNTS) for p in (0, 3, 4, 5)}
    for p, t in tables.items():
        t.set_option(px.OPT_NONTEMPORAL, p)
    g = [_gauss(981, w) for w in range(2)]
    want = oracle_mod.reduce_avg_tensors(g, np.float16)
    for p, t in tables.items():
        d_out = empty_like_device(COUNTS, np.float16)
        px.reduce_avg(t, [t.bufset(to_device(x)) for x in g], t.bufset(d_out))
        assert_bits_equal(to_host(d_out), want, f"table under policy {p}")
        assert t.get_option(px.OPT_NONTEMPORAL) == p
    assert px.get_option(px.OPT_NONTEMPORAL) == -1
