"""pxchg_buffer_stats_static, the diagnostics call that allocates nothing (its partial results live in a static
device array of the library): through the C ABI, against pxchg_buffer_stats and the oracle, bit for bit, on two
calls in a row of which the second has the smaller input, so that the array still holds the first call's partial
results when the second one runs."""
import os
import re

import numpy as np
import pytest

import workloads as wl
from gpu_util import to_device

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def px():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1605_08325_amd as px
    px.load()
    return px


def header_constant(name):
    text = open(os.path.join(ROOT, "include", "pxchg.h")).read()
    return int(re.search(rf"#define\s+{name}\s+(\d+)", text).group(1))


def oracle_stats(oracle_mod, tensors):
    return oracle_mod.stats_ordered_tensors(tensors, 512, header_constant("PXCHG_STATS_WAVES"),
                                            header_constant("PXCHG_STATS_BLOCK_CHUNKS"),
                                            header_constant("PXCHG_STATS_COMBINE_THREADS"))


@pytest.mark.parametrize("dt", [np.float16, np.float32])
def test_static_scratch_call_equals_the_regular_call_twice_in_a_row(px, oracle_mod, dt):
    import torch
    big_counts = [34_848, 96, 3_000_001, 0, 70_001, 8192 * 40 + 5]     # 54 blocks of partial results
    small_counts = [20_001, 3, 513]                                     # 1 block
    results = []
    for counts, seed in ((big_counts, 31), (small_counts, 32)):
        a = [t.astype(dt) for t in wl.gaussian_tensors(counts, 0.01, seed, "grad")]
        a[0][7] = np.inf
        a[-1][-1] = -3.5
        table = px.Table(counts)
        s = table.bufset(to_device(a))
        out_static = torch.full((3,), -1, dtype=torch.int64, device="cuda")
        out_regular = torch.full((3,), -1, dtype=torch.int64, device="cuda")
        px.buffer_stats_static(table, s, out_static)
        px.buffer_stats(table, s, out_regular)
        torch.cuda.synchronize()
        got, want = px.read_stats(out_static), px.read_stats(out_regular)
        assert got == want, (counts, got, want)
        assert got == oracle_stats(oracle_mod, a)
        assert got[0] == 1 and got[1] == 3.5
        results.append(got)
    assert results[0] != results[1]
    # and once more on the first size, after the smaller call: nothing stale is picked up
    a = [t.astype(dt) for t in wl.gaussian_tensors(big_counts, 0.01, 33, "grad")]
    table = px.Table(big_counts)
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    px.buffer_stats_static(table, table.bufset(to_device(a)), out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == oracle_stats(oracle_mod, a)


def test_static_scratch_call_through_a_view_and_on_an_empty_table(px, oracle_mod):
    import torch
    counts = [5000, 0, 8192 * 9 + 1, 700]
    a = wl.gaussian_tensors(counts, 0.01, 34, "grad")
    table = px.Table(counts)
    s = table.bufset(to_device(a))
    out = torch.zeros(3, dtype=torch.int64, device="cuda")
    px.buffer_stats_static(table.view(2, 2), s, out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == oracle_stats(oracle_mod, a[2:4])
    empty = px.Table([0, 0])
    out.fill_(-1)
    px.buffer_stats_static(empty, px.BufSet(empty, [0, 0], px.F16), out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == (0, 0.0, 0.0)


def test_static_scratch_call_refuses_what_does_not_fit(px):
    """One chunk more than the static array has room for (in blocks of chunks): PXCHG_ERR_UNSUPPORTED, nothing
    launched, the output untouched; the regular call takes the same table."""
    import torch
    limit = header_constant("PXCHG_STATS_STATIC_MAX_BLOCKS") * header_constant("PXCHG_STATS_BLOCK_CHUNKS")
    n = limit * 512 + 1
    table = px.Table([n])
    assert table.n_chunks == limit + 1
    data = torch.zeros(n, dtype=torch.float16, device="cuda")           # 1 GiB
    data[-1] = 2.0
    s = table.bufset([data])
    out = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    with pytest.raises(px.PxchgError) as e:
        px.buffer_stats_static(table, s, out)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert out.tolist() == [-1, -1, -1]
    px.buffer_stats(table, s, out)
    torch.cuda.synchronize()
    assert px.read_stats(out) == (0, 2.0, 4.0)
    del data
    torch.cuda.empty_cache()
