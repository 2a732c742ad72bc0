"""GPU parity on the five benchmark configurations at their full sizes, in the
default launch configuration (the one bench.py times).  Every configuration is
compared with the oracle on EVERY element at least once (one whole step, or one
whole elastic round).  The multi-step loops then go on against the oracle on a
fixed sample of elements per tensor (the operations are element-wise, so the
oracle run on the gathered sample is the same arithmetic; the sample always
includes each tensor's first and last elements and the elements around chunk
boundaries), and their final state is compared on every element, GPU against
GPU, with the same loop run through the library's other code path (fused
reduce+update against the two calls, k single meetings against fused rounds)."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import assert_bits_equal, assert_close_params, empty_like_device, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def px():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1605_08325_amd as px
    px.load()
    return px


def sample_indices(counts, per_tensor, seed, chunk):
    rng = np.random.default_rng(seed)
    out = []
    for c in counts:
        if c <= per_tensor:
            out.append(np.arange(c))
            continue
        idx = [rng.integers(0, c, per_tensor), np.arange(0, 64), np.arange(c - 64, c)]
        for b in range(chunk, c, chunk * max(1, (c // chunk) // 16)):     # around some chunk boundaries
            idx.append(np.arange(max(0, b - 16), min(c, b + 16)))
        out.append(np.unique(np.concatenate(idx)))
    return out


def gather(tensors, idx):
    return [np.ascontiguousarray(t[i]) for t, i in zip(tensors, idx)]


def gather_device(tensors, idx):
    import torch
    return [t[torch.from_numpy(i).to("cuda")].cpu().numpy() for t, i in zip(tensors, idx)]


def sync_exchange(px, oracle_mod, cfg, steps, full):
    """pack (if half-precision transfer) -> reduce+average -> update, `steps` times."""
    import torch
    counts = list(cfg.counts)
    table = px.Table(counts)
    half = cfg.transfer == "f16"
    wire = np.float16 if half else np.float32
    w = [a.copy() for a in wl.gaussian_tensors(counts, cfg.param_sigma, cfg.seed, "param")]
    v = wl.zeros_tensors(counts)
    d_w, d_v = to_device(w), to_device(v)
    sw, sv = table.bufset(d_w), table.bufset(d_v)
    d_avg = empty_like_device(counts, wire)
    s_avg = table.bufset(d_avg)
    twin = steps > 1          # a second copy of the state, stepped by the fused call: compared on every element
    if twin:
        d_w2, d_v2 = to_device(w), to_device(v)
        sw2, sv2 = table.bufset(d_w2), table.bufset(d_v2)
    idx = None if full else sample_indices(counts, 20_000, cfg.seed, px.get_option(px.OPT_CHUNK_ELEMS))
    if idx is not None:
        w, v = gather(w, idx), gather(v, idx)
    for step in range(steps):
        grads = wl.gaussian_workers(counts, cfg.grad_sigma, cfg.seed, "grad", cfg.k, step)
        d_g = [to_device(g) for g in grads]
        s_g = [table.bufset(g) for g in d_g]
        if half:
            d_h = [empty_like_device(counts, np.float16) for _ in range(cfg.k)]
            s_h = [table.bufset(h) for h in d_h]
            px.pack_fp16(table, s_g, s_h)
            contrib_sets = s_h
        else:
            contrib_sets = s_g
        px.reduce_avg(table, contrib_sets, s_avg)
        px.sgd_momentum(table, s_avg, sw, sv, cfg.lr, cfg.mu, cfg.wd)
        if twin:
            px.reduce_avg_sgd_momentum(table, contrib_sets, sw2, sv2, cfg.lr, cfg.mu, cfg.wd, px.AVG,
                                       px.F16 if half else px.F32)
        torch.cuda.synchronize()
        # oracle on all elements, or on the gathered sample
        if idx is not None:
            grads = [gather(g, idx) for g in grads]
        contrib = [oracle_mod.pack_fp16_tensors(g) for g in grads] if half else grads
        if half and step == 0:
            for i in (0, cfg.k - 1):
                got = to_host(d_h[i]) if idx is None else gather_device(d_h[i], idx)
                assert_bits_equal(got, contrib[i], f"{cfg.name} packed worker {i}")
        avg = oracle_mod.reduce_avg_tensors(contrib, wire)
        got = to_host(d_avg) if idx is None else gather_device(d_avg, idx)
        assert_bits_equal(got, avg, f"{cfg.name} average step {step}")
        oracle_mod.sgd_momentum_tensors(avg, w, v, cfg.lr, cfg.mu, cfg.wd)
        del d_g, s_g
    got_w = to_host(d_w) if idx is None else gather_device(d_w, idx)
    got_v = to_host(d_v) if idx is None else gather_device(d_v, idx)
    assert_close_params(got_w, w, cfg.name)          # the stated tolerance
    assert_bits_equal(got_w, w, f"{cfg.name} params")  # and in fact bit-exact
    assert_bits_equal(got_v, v, f"{cfg.name} velocity")
    if twin:
        for t in range(len(counts)):
            assert torch.equal(d_w[t].view(torch.int32), d_w2[t].view(torch.int32)), f"{cfg.name} fused twin, w[{t}]"
            assert torch.equal(d_v[t].view(torch.int32), d_v2[t].view(torch.int32)), f"{cfg.name} fused twin, v[{t}]"


def test_config1_tiny_sync(px, oracle_mod):
    sync_exchange(px, oracle_mod, wl.config(1), steps=1, full=True)


def test_config2_alexnet_k2_f32(px, oracle_mod):
    sync_exchange(px, oracle_mod, wl.config(2), steps=1, full=True)


def test_config3_alexnet_k8_f16_one_step_all_elements(px, oracle_mod):
    sync_exchange(px, oracle_mod, wl.config(3), steps=1, full=True)


def test_config3_alexnet_k8_f16_ten_steps_sampled(px, oracle_mod):
    cfg = wl.config(3)
    sync_exchange(px, oracle_mod, cfg, steps=cfg.steps, full=False)


def test_config4_many_small_tensors_one_launch_per_stage(px, oracle_mod):
    cfg = wl.config(4)
    assert len(cfg.counts) == 116 and cfg.n == 7_000_000
    sync_exchange(px, oracle_mod, cfg, steps=2, full=True)


def test_config5_easgd_100_rounds(px, oracle_mod):
    """Round 1 on every element against the oracle (single meetings, and the fused round on a second copy of the
    state); all 100 rounds against the oracle on the sample; after the last round the two copies, one stepped by
    single meetings and fused rounds half and half, the other the other way round, agree on every element."""
    import torch
    cfg = wl.config(5)
    counts = list(cfg.counts)
    table = px.Table(counts)
    xs = [[a.copy() for a in x] for x in wl.gaussian_workers(counts, cfg.param_sigma, cfg.seed, "worker", cfg.k)]
    c = [a.copy() for a in wl.gaussian_tensors(counts, cfg.param_sigma, cfg.seed, "center")]
    d_xs, d_c = [to_device(x) for x in xs], to_device(c)
    d_xs2, d_c2 = [to_device(x) for x in xs], to_device(c)
    s_xs, s_c = [table.bufset(x) for x in d_xs], table.bufset(d_c)
    s_xs2, s_c2 = [table.bufset(x) for x in d_xs2], table.bufset(d_c2)
    orders = wl.worker_orders(cfg.seed, cfg.k, cfg.rounds)
    alpha = np.float32(cfg.alpha)

    def meetings(sets, center, order):
        for i in order:
            px.easgd(table, sets[i], center, float(alpha))

    def fused(sets, center, order):
        px.easgd_round(table, [sets[i] for i in order], center, float(alpha))

    # round 1, every element
    meetings(s_xs, s_c, orders[0])
    fused(s_xs2, s_c2, orders[0])
    for i in orders[0]:
        oracle_mod.easgd_tensors(xs[i], c, alpha)
    torch.cuda.synchronize()
    for i in range(cfg.k):
        assert_bits_equal(to_host(d_xs[i]), xs[i], f"round 1, worker {i}, single meetings")
        assert_bits_equal(to_host(d_xs2[i]), xs[i], f"round 1, worker {i}, fused round")
    assert_bits_equal(to_host(d_c), c, "round 1, center, single meetings")
    assert_bits_equal(to_host(d_c2), c, "round 1, center, fused round")

    # rounds 2..100 against the oracle on the sample
    idx = sample_indices(counts, 20_000, cfg.seed, px.get_option(px.OPT_CHUNK_ELEMS))
    xs = [gather(x, idx) for x in xs]
    c = gather(c, idx)
    for r, order in enumerate(orders):
        if r == 0:
            continue
        first_half = r < cfg.rounds // 2
        (meetings if first_half else fused)(s_xs, s_c, order)
        (fused if first_half else meetings)(s_xs2, s_c2, order)
        for i in order:
            oracle_mod.easgd_tensors(xs[i], c, alpha)
    torch.cuda.synchronize()
    for i in range(cfg.k):
        got = gather_device(d_xs[i], idx)
        assert_close_params(got, xs[i], f"worker {i}")
        assert_bits_equal(got, xs[i], f"worker {i}")
    assert_bits_equal(gather_device(d_c, idx), c, "center")
    for t in range(len(counts)):
        assert torch.equal(d_c[t].view(torch.int32), d_c2[t].view(torch.int32)), f"center[{t}], the two paths"
        for i in range(cfg.k):
            assert torch.equal(d_xs[i][t].view(torch.int32), d_xs2[i][t].view(torch.int32)), f"worker {i}[{t}], the two paths"


# ------------------------------------------------------------------ the paper's other two model sizes (Table 2)

def test_vggnet_shaped_k8_f16_one_step_all_elements(px, oracle_mod):
    """138,357,544 parameters in 32 tensors (Table 2's VGGNet count), same exchange as configuration 3, every
    element against the oracle."""
    base = wl.config(3)
    cfg = wl.Config("vggnet_sync_k8_f16", tuple(wl.vggnet_counts()), 8, "f16", seed=base.seed + 100)
    sync_exchange(px, oracle_mod, cfg, steps=1, full=True)


def test_googlenet_count_many_small_tensors_k8_f16(px, oracle_mod):
    """13,378,280 parameters (Table 2's GoogLeNet count) spread over 128 ragged tensors."""
    base = wl.config(4)
    cfg = wl.Config("googlenet_sync_k8_f16", tuple(wl.googlenet_scale_counts(base.seed)), 8, "f16",
                    seed=base.seed + 100)
    sync_exchange(px, oracle_mod, cfg, steps=1, full=True)


def test_weight_averaging_mode_on_alexnet_shapes(px, oracle_mod):
    """Section 4's other scheme: every worker descends on its own (learning rate scaled by k), then weights
    and momentum are averaged (binary32 transfer, k = 8).  Same kernels, no update after the average."""
    import torch
    cfg = wl.config(2)
    counts, k = list(cfg.counts), 8
    table = px.Table(counts)
    idx = sample_indices(counts, 20_000, cfg.seed, px.get_option(px.OPT_CHUNK_ELEMS))
    w0 = wl.gaussian_tensors(counts, cfg.param_sigma, cfg.seed, "param")
    grads = wl.gaussian_workers(counts, cfg.grad_sigma, cfg.seed, "grad", k)
    d_ws = [to_device(w0) for _ in range(k)]
    d_vs = [to_device(wl.zeros_tensors(counts)) for _ in range(k)]
    s_ws, s_vs = [table.bufset(w) for w in d_ws], [table.bufset(v) for v in d_vs]
    for i in range(k):
        px.sgd_momentum(table, table.bufset(to_device(grads[i])), s_ws[i], s_vs[i], k * cfg.lr, cfg.mu, cfg.wd)
    px.reduce_avg(table, s_ws, s_ws[0])        # in place into worker 0's copy
    px.reduce_avg(table, s_vs, s_vs[0])
    torch.cuda.synchronize()
    ws, vs = [], []
    for i in range(k):
        wi, vi = gather(w0, idx), gather(wl.zeros_tensors(counts), idx)
        oracle_mod.sgd_momentum_tensors(gather(grads[i], idx), wi, vi, np.float32(k * cfg.lr), cfg.mu, cfg.wd)
        ws.append(wi)
        vs.append(vi)
    assert_bits_equal(gather_device(d_ws[0], idx), oracle_mod.reduce_avg_tensors(ws), "averaged weights")
    assert_bits_equal(gather_device(d_vs[0], idx), oracle_mod.reduce_avg_tensors(vs), "averaged momentum")
