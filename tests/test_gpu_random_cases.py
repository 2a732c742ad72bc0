"""Seeded random cases of every call against the oracle: tensor counts around chunk and vector boundaries, every
operand at its own misalignment, any worker count, both element types, the two cache policies of the regular build and two chunk sizes.
The cases are drawn from a fixed seed, so a failure names a case that can be run again."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_bits_equal, to_device, to_host

pytestmark = pytest.mark.gpu

N_CASES = 60


@pytest.fixture(scope="module")
def px():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1605_08325_amd as px
    px.load()
    return px


def _counts(rng):
    out = []
    for _ in range(int(rng.integers(1, 6))):
        kind = rng.integers(0, 5)
        if kind == 0:
            out.append(int(rng.integers(0, 20)))
        elif kind == 1:
            out.append(int(rng.integers(1, 5)) * 512 + int(rng.integers(-9, 10)))
        elif kind == 2:
            out.append(int(rng.integers(1, 4)) * 1024 + int(rng.integers(-3, 4)))
        else:
            out.append(int(rng.integers(20, 6000)))
    return out


def _draw(rng, counts, dtype, scale=0.01):
    return [(rng.standard_normal(c) * scale).astype(dtype) for c in counts]


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_case(px, oracle_mod, case):
    rng = np.random.default_rng(wl.BASE_SEED * 1000 + case)
    counts = _counts(rng)
    k = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 12]))
    in_dt, out_dt = (np.float32, np.float16)[int(rng.integers(2))], (np.float32, np.float16)[int(rng.integers(2))]
    policy = int(rng.integers(-1, 6))
    policy = policy if policy <= 0 else -(policy % 2)   # the regular build: each kernel's own policy (-1) or plain (0)
    chunk = int(rng.choice([512, 1024]))
    same_offset = bool(rng.integers(2))
    base_off = int(rng.integers(0, 8))
    off = (lambda: base_off) if same_offset else (lambda: int(rng.integers(0, 8)))
    lr, mu, wd, alpha = 0.01, 0.9, float(rng.choice([0.0, 5e-4])), float(rng.choice([0.0625, 0.1, 0.5]))
    mode = int(rng.integers(2))
    print(f"case {case}: counts={counts} k={k} in={np.dtype(in_dt).name} out={np.dtype(out_dt).name} "
          f"policy={policy} chunk={chunk} same_offset={same_offset} wd={wd} alpha={alpha} mode={mode}", flush=True)
    old = (px.get_option(px.OPT_CHUNK_ELEMS), px.get_option(px.OPT_NONTEMPORAL), px.get_option(px.OPT_CENTER_RESIDENT))
    try:
        px.set_option(px.OPT_CHUNK_ELEMS, chunk)
        px.set_option(px.OPT_NONTEMPORAL, policy)
        px.set_option(px.OPT_CENTER_RESIDENT, int(rng.integers(2)))
        table = px.Table(counts)
        # pack and unpack
        g = [_draw(rng, counts, np.float32) for _ in range(k)]
        d_h = [to_device([np.zeros(c, np.float16) for c in counts], off()) for _ in range(k)]
        s_h = [table.bufset(t) for t in d_h]
        px.pack_fp16(table, [table.bufset(to_device(t, off())) for t in g], s_h)
        packed = [oracle_mod.pack_fp16_tensors(t) for t in g]
        for i in range(k):
            assert_bits_equal(to_host(d_h[i]), packed[i], f"pack {i}")
        d_back = to_device([np.zeros(c, np.float32) for c in counts], off())
        px.unpack_fp16(table, [s_h[0]], [table.bufset(d_back)])
        assert_bits_equal(to_host(d_back), oracle_mod.unpack_fp16_tensors(packed[0]), "unpack")
        # reduce
        contrib = [[a.astype(in_dt) for a in t] for t in g]
        s_c = [table.bufset(to_device(t, off())) for t in contrib]
        d_out = to_device([np.zeros(c, out_dt) for c in counts], off())
        s_out = table.bufset(d_out)
        px.reduce_avg(table, s_c, s_out, mode)
        avg = oracle_mod.reduce_avg_tensors(contrib, out_dt, mode)
        assert_bits_equal(to_host(d_out), avg, "reduce")
        # update, staged and fused
        w, v = _draw(rng, counts, np.float32, 0.05), _draw(rng, counts, np.float32, 0.001)
        w2, v2 = [a.copy() for a in w], [a.copy() for a in v]
        d_w, d_v = to_device(w, off()), to_device(v, off())
        px.sgd_momentum(table, s_out, table.bufset(d_w), table.bufset(d_v), lr, mu, wd)
        oracle_mod.sgd_momentum_tensors(avg, w, v, lr, mu, wd)
        assert_bits_equal(to_host(d_w), w, "w")
        assert_bits_equal(to_host(d_v), v, "v")
        d_w2, d_v2 = to_device(w2, off()), to_device(v2, off())
        wire = px.F16 if out_dt == np.float16 else px.F32
        px.reduce_avg_sgd_momentum(table, s_c, table.bufset(d_w2), table.bufset(d_v2), lr, mu, wd, mode, wire)
        assert_bits_equal(to_host(d_w2), w, "fused w")
        assert_bits_equal(to_host(d_v2), v, "fused v")
        # elastic: a fused round, then one more meeting of the last worker
        xs = [_draw(rng, counts, np.float32) for _ in range(k)]
        c = _draw(rng, counts, np.float32)
        d_xs, d_c = [to_device(x, off()) for x in xs], to_device(c, off())
        s_xs, s_cc = [table.bufset(t) for t in d_xs], table.bufset(d_c)
        px.easgd_round(table, s_xs, s_cc, alpha)
        px.easgd(table, s_xs[k - 1], s_cc, alpha)
        for i in list(range(k)) + [k - 1]:
            oracle_mod.easgd_tensors(xs[i], c, np.float32(alpha))
        for i in range(k):
            assert_bits_equal(to_host(d_xs[i]), xs[i], f"x[{i}]")
        assert_bits_equal(to_host(d_c), c, "center")
        # diagnostics of the average
        import torch
        out = torch.zeros(3, dtype=torch.int64, device="cuda")
        px.buffer_stats(table, s_out, out)
        torch.cuda.synchronize()
        bad, mx, ss = px.read_stats(out)
        wbad, wmx, wss = oracle_mod.stats_tensors(avg)
        assert (bad, mx) == (wbad, wmx) and abs(ss - wss) <= 1e-12 * max(wss, 1e-300)
    finally:
        px.set_option(px.OPT_CHUNK_ELEMS, old[0])
        px.set_option(px.OPT_NONTEMPORAL, old[1])
        px.set_option(px.OPT_CENTER_RESIDENT, old[2])
