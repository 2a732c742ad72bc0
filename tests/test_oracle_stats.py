"""Pins for the oracle's tree-ordered diagnostics (oracle_stats_ordered): the sum of squares in the fixed order
that the library's header defines, so that a GPU can reproduce it bit for bit.

The hand cases use one large element whose square B has an ulp of 4 units of the small elements' squares, so that
which accumulator a small element lands in (same lane as the large one: lost to rounding one at a time; another
lane, wavefront or block: added up first and kept) decides the result.  Every expected value is derived from the
definition by hand and written as literal binary64 arithmetic; nothing here re-implements the tree."""
import math

import numpy as np
import pytest

BIG32 = np.float32(2.0 ** 27)       # square 2^54: binary64 ulp 4, so +1 is lost and +2 is a tie that goes to even
B = 2.0 ** 54
BIG16 = np.float16(2.0 ** 15)       # square 2^30: binary64 ulp 2^-22
SMALL16 = np.float16(2.0 ** -12)    # square 2^-24, a quarter of that ulp


def ordered(oracle_mod, ts, chunk=512, waves=4, block=8, threads=256):
    return oracle_mod.stats_ordered_tensors(ts, chunk, waves, block, threads)


def f32(n, **at):
    a = np.zeros(n, np.float32)
    for i, v in at.items():
        a[int(i[1:])] = v
    return a


def with_ones(n, big_at, ones_at):
    a = np.zeros(n, np.float32)
    a[big_at] = BIG32
    a[list(ones_at)] = 1.0
    return a


def test_the_rounding_facts_the_hand_cases_rest_on():
    assert B + 1.0 == B and B + 2.0 == B and B + 3.0 == B + 4.0 and B + 4.0 != B
    assert float(BIG32) ** 2 == B and float(BIG16) ** 2 == 2.0 ** 30 and float(SMALL16) ** 2 == 2.0 ** -24
    assert 2.0 ** 30 + 2.0 ** -24 == 2.0 ** 30 and 2.0 ** 30 + 2.0 ** -21 != 2.0 ** 30


def test_lane_of_an_element_is_its_16_byte_piece_modulo_64(oracle_mod):
    # binary32: pieces of 4.  Elements 1..3 share lane 0 with the large one (each +1 is lost); 4..7 are lane 1
    # (they add up to 4 there and meet lane 0 in the last butterfly step).
    assert ordered(oracle_mod, [with_ones(512, 0, range(1, 4))])[2] == B
    assert ordered(oracle_mod, [with_ones(512, 0, range(4, 8))])[2] == B + 4.0
    assert ordered(oracle_mod, [with_ones(512, 0, range(1, 8))])[2] == B + 4.0
    # piece 64 is lane 0 again
    assert ordered(oracle_mod, [with_ones(512, 0, range(256, 260))])[2] == B
    assert ordered(oracle_mod, [with_ones(512, 0, range(252, 256))])[2] == B + 4.0
    # binary16: pieces of 8.  1..7 are lane 0 (lost), 8..15 lane 1 (8 x 2^-24 = 2^-21, kept)
    h = np.zeros(512, np.float16)
    h[0] = BIG16
    h[1:8] = SMALL16
    assert ordered(oracle_mod, [h])[2] == 2.0 ** 30
    h[8:16] = SMALL16
    assert ordered(oracle_mod, [h])[2] == 2.0 ** 30 + 2.0 ** -21
    # the index order (what oracle_stats does) loses all of them, one at a time
    assert oracle_mod.stats(h)[2] == 2.0 ** 30


def test_wave_of_a_chunk_is_its_place_in_the_block_modulo_waves(oracle_mod):
    # 4 chunks of 512 in one block, 2 waves: chunks 0 and 2 are wave 0, chunks 1 and 3 wave 1
    kw = dict(chunk=512, waves=2, block=4, threads=64)
    assert ordered(oracle_mod, [with_ones(2048, 0, range(1024, 1028))], **kw)[2] == B         # chunk 2, lane 0: same accumulator
    assert ordered(oracle_mod, [with_ones(2048, 0, range(512, 516))], **kw)[2] == B + 4.0     # chunk 1: wave 1
    assert ordered(oracle_mod, [with_ones(2048, 0, range(1536, 1540))], **kw)[2] == B + 4.0   # chunk 3: wave 1
    # with 4 waves chunk 2 has a wave of its own
    assert ordered(oracle_mod, [with_ones(2048, 0, range(1024, 1028))], chunk=512, waves=4, block=4, threads=64)[2] == B + 4.0


def test_blocks_are_runs_of_block_chunks_chunks(oracle_mod):
    a = with_ones(2048, 0, range(1024, 1028))                  # the ones sit in chunk 2
    assert ordered(oracle_mod, [a], chunk=512, waves=2, block=4, threads=64)[2] == B          # same block, same accumulator
    assert ordered(oracle_mod, [a], chunk=512, waves=2, block=2, threads=64)[2] == B + 4.0    # chunk 2 opens block 1
    # a last, incomplete block still counts
    assert ordered(oracle_mod, [a[:1030]], chunk=512, waves=2, block=2, threads=64)[2] == B + 4.0


def test_chunks_never_straddle_tensors(oracle_mod):
    # tensor 1 starts a new chunk (wave 1, lane 0), wherever tensor 0 ended
    ts = [np.array([BIG32], np.float32), np.ones(4, np.float32)]
    assert ordered(oracle_mod, ts, chunk=512, waves=2, block=2, threads=64)[2] == B + 4.0
    flat = np.concatenate(ts)                                   # one tensor: 1..3 are lane 0, 4 is lane 1 (a lone 1, lost)
    assert ordered(oracle_mod, [flat], chunk=512, waves=2, block=2, threads=64)[2] == B
    # empty tensors give no chunk, so they do not shift the wave of what follows
    ts2 = [ts[0], np.zeros(0, np.float32), np.zeros(0, np.float32), ts[1]]
    assert ordered(oracle_mod, ts2, chunk=512, waves=2, block=2, threads=64)[2] == B + 4.0


def test_butterfly_pairs_lane_l_with_l_xor_32_first(oracle_mod):
    # lanes 1 and 33 hold 2 each: the first step (off 32) makes 4 of them, the last (off 1) brings it to lane 0
    a = with_ones(512, 0, [4, 5, 33 * 4, 33 * 4 + 1])
    assert ordered(oracle_mod, [a])[2] == B + 4.0
    # lanes 1 and 2 hold 2 each: lane 2 reaches lane 0 in step off 2 (a tie, lost), lane 1 in step off 1 (lost)
    a = with_ones(512, 0, [4, 5, 8, 9])
    assert ordered(oracle_mod, [a])[2] == B
    # lanes 1 and 3: they meet in step off 2 (lane 1 = 2 + 2), kept
    a = with_ones(512, 0, [4, 5, 12, 13])
    assert ordered(oracle_mod, [a])[2] == B + 4.0


def test_waves_are_added_in_order_starting_from_wave_0(oracle_mod):
    kw = dict(chunk=512, waves=4, block=4, threads=64)
    a = with_ones(2048, 0, [512, 513, 1024, 1025])              # wave 1 and wave 2 hold 2 each
    assert ordered(oracle_mod, [a], **kw)[2] == B                # (B + 2) + 2: two ties, both lost
    a = with_ones(2048, 512, [0, 1, 1024, 1025])                # the large one in wave 1: (2 + B) + 2
    assert ordered(oracle_mod, [a], **kw)[2] == B
    a = with_ones(2048, 1024, [0, 1, 512, 513])                 # the large one in wave 2: (2 + 2) + B
    assert ordered(oracle_mod, [a], **kw)[2] == B + 4.0


def test_final_combine_gives_block_b_to_thread_b_modulo_threads(oracle_mod):
    # one chunk of 8 elements per block, 64 combine threads: blocks 0, 64, 128, ... all go to thread 0 in turn
    kw = dict(chunk=8, waves=1, block=1, threads=64)
    n_blocks = 257
    a = np.zeros(8 * n_blocks, np.float32)
    a[0] = BIG32
    a[[8 * 64, 8 * 128, 8 * 192, 8 * 256]] = 1.0
    assert ordered(oracle_mod, [a], **kw)[2] == B                # thread 0: ((((B + 1) + 1) + 1) + 1)
    a[:] = 0
    a[0] = BIG32
    a[[8 * 1, 8 * 65, 8 * 129, 8 * 193]] = 1.0                  # thread 1 collects 4, meets thread 0 in the last step
    assert ordered(oracle_mod, [a], **kw)[2] == B + 4.0
    # with 128 threads, blocks 64 and 192 belong to thread 64 (second group), 128 and 256 to thread 0
    a[:] = 0
    a[0] = BIG32
    a[[8 * 64, 8 * 192, 8 * 64 + 1, 8 * 192 + 1]] = 1.0         # 4 in thread 64: group 1's value, added to group 0's
    assert ordered(oracle_mod, [a], chunk=8, waves=1, block=1, threads=128)[2] == B + 4.0
    assert ordered(oracle_mod, [a], **kw)[2] == B


@pytest.mark.parametrize("dt", [np.float32, np.float16])
@pytest.mark.parametrize("params", [(512, 4, 64, 1024), (512, 16, 32, 256), (2048, 3, 5, 64), (7, 2, 3, 128)])
def test_any_order_is_exact_on_small_integers(oracle_mod, dt, params):
    rng = np.random.default_rng(5)
    counts = [1, 0, 700, 513, 4096 + 3, 20_000]
    ts = [rng.integers(-30, 31, c).astype(dt) for c in counts]
    want = sum(int(v) ** 2 for t in ts for v in t.astype(np.int64))
    bad, mx, ss = oracle_mod.stats_ordered_tensors(ts, *params)
    assert (bad, ss) == (0, float(want)) and mx == max(float(np.max(np.abs(t))) for t in ts if t.size)
    assert oracle_mod.stats_tensors(ts)[2] == float(want)


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_against_the_exactly_rounded_sum_and_numpy(oracle_mod, dt):
    rng = np.random.default_rng(6)
    counts = [3, 65, 70_001, 8192, 300_000]
    ts = [(rng.standard_normal(c) * 0.01).astype(dt) for c in counts]
    ts[2][[5, 69_000]] = [np.inf, np.nan]
    ts[4][7] = -np.inf
    n = sum(counts)
    bad, mx, ss = oracle_mod.stats_ordered_tensors(ts, 512, 4, 64, 1024)
    finite = [t[np.isfinite(t)].astype(np.float64) for t in ts]
    exact = math.fsum(float(v) * float(v) for t in finite for v in t)      # squares exact, sum exactly rounded
    assert bad == 3 and mx == max(float(np.max(np.abs(t))) for t in finite)
    # a tree of binary64 additions of n non-negative terms: each term passes through at most
    # log2(n) + a few roundings, far fewer than the n - 1 of the index-order sum
    assert abs(ss - exact) <= 64 * 2.0 ** -53 * exact
    assert abs(oracle_mod.stats_tensors(ts)[2] - exact) <= n * 2.0 ** -53 * exact
    assert ss != 0.0


def test_special_cases(oracle_mod):
    assert ordered(oracle_mod, [np.zeros(0, np.float32)]) == (0, 0.0, 0.0)
    assert ordered(oracle_mod, [np.array([np.nan, np.inf, -np.inf], np.float32)]) == (3, 0.0, 0.0)
    # an element that is not finite adds nothing and keeps its place: the ones after it stay in their lanes
    a = with_ones(512, 0, range(4, 8))
    a[1] = np.nan
    assert ordered(oracle_mod, [a]) == (1, float(BIG32), B + 4.0)
    # negative values, zeros of both signs, the smallest subnormal
    tiny = np.array([-0.0, 1e-45, -3.0], np.float32)
    assert ordered(oracle_mod, [tiny]) == (0, 3.0, 9.0)       # 1e-90 is far below half an ulp of 9
    with pytest.raises(ValueError):
        oracle_mod.stats_ordered_tensors([tiny], 512, 4, 64, 100)     # combine threads must be whole groups of 64
    with pytest.raises(ValueError):
        oracle_mod.stats_ordered_tensors([tiny], 0, 4, 64, 128)
