#!/usr/bin/env python3
"""Benchmark of the parameter-exchange hot path on one MI355X.

Workload: the AlexNet-shaped half-precision exchange with k = 8 workers
(60,965,224 float32 parameters in 16 separately allocated tensors).  One step is
one pass of the whole path over one batch of synthetic gradients:

    pack      8 workers' float32 gradients -> binary16              (1 launch)
    reduce    fixed-order float32 sum of the 8 halves, /8, -> half  (1 launch)
    update    momentum SGD with the half-precision average          (1 launch)
    elastic   one asynchronous round: 8 workers meet the center     (8 launches)

Everything is resident in HBM before the timed region.  The headline value is
the metric the build is graded on: reduce+update GB/s = algorithmic bytes of the
two stages (2k+2 and 18 bytes per element) over their measured time.  Stage
times come from HIP events recorded on the launch stream between the stages of
every timed step; the `roofline` object is for the kernel with the largest share
of the step, `stages` lists all of them.

`extras` holds what is measured after the timed region, each over the same number
of repetitions: the fused reduce+update and the fused elastic round, the elastic
kernels with the center kept in the memory-side cache, the diagnostics pass, the
same reduce+update issued layer by layer on two streams, the whole step replayed
from a HIP graph, and weight averaging (the reduce over float32 sets).

`cpu_baseline` is the CPU oracle timed on the host cores on the same workload.
It is a reported baseline (and the only place this program touches the oracle),
never a fallback: without the built HIP library this program fails.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak

# HBM traffic per launch from hardware counters (FETCH_SIZE + WRITE_SIZE, scaled by
# what the same counters read for a plain copy of known size); see the files named.
MEASURED_TRAFFIC_BYTES = {
    # stage: (bytes per launch, profile summary it comes from)
    "pack": (2_925_961_070, "profiles/bench_alexnet_k8_hbm_counters.txt"),
    "reduce": (1_054_182_083, "profiles/bench_alexnet_k8_hbm_counters.txt"),
    "update": (1_075_740_713, "profiles/bench_alexnet_k8_hbm_counters.txt"),
    "elastic": (960_996_176, "profiles/bench_alexnet_k8_hbm_counters.txt"),
}


def host_threads() -> int:
    n = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, min(n, 16))


def upload(tensors):
    import torch
    return [torch.from_numpy(np.ascontiguousarray(a)).to("cuda") for a in tensors]


def cpu_baseline(counts, grads, w, v, xs, c, order, cfg, alpha, threads):
    """The oracle, as it stands, on the host cores: same stages, same inputs.  Returns per-stage seconds with
    all `threads` host threads (element range split over them) and with one thread."""
    import ctypes

    import oracle
    L = oracle.lib()
    k = len(grads)
    half = cfg.transfer == "f16"
    flat = lambda ts: np.concatenate(ts) if len(ts) > 1 else ts[0].copy()  # noqa: E731
    # one flat copy per buffer: the oracle is element-wise, so flattening the
    # tensor list changes nothing but the loop bounds
    g = [flat(t) for t in grads]
    n = g[0].size
    wire = np.float16 if half else np.float32
    wire_es, wire_id = (2, oracle.F16) if half else (4, oracle.F32)
    h = [np.empty(n, np.float16) for _ in range(k)] if half else g
    avg = np.empty(n, wire)
    wf, vf = flat(w), flat(v)
    xf, cf = [flat(t) for t in xs], flat(c)

    def ptr(a, off, es):
        return ctypes.c_void_p(a.ctypes.data + off * es)

    def pack(span):
        a, b = span
        for i in range(k):
            L.oracle_pack_fp16(ptr(g[i], a, 4), ptr(h[i], a, 2), b - a)

    def reduce(span):
        a, b = span
        ps = (ctypes.c_void_p * k)(*[h[i].ctypes.data + a * wire_es for i in range(k)])
        L.oracle_reduce_avg(k, ps, wire_id, ptr(avg, a, wire_es), wire_id, oracle.AVG, b - a)

    def update(span):
        a, b = span
        L.oracle_sgd_momentum(ptr(avg, a, wire_es), wire_id, ptr(wf, a, 4), ptr(vf, a, 4),
                              cfg.lr, cfg.mu, cfg.wd, b - a)

    def elastic(span):
        a, b = span
        for i in order:
            L.oracle_easgd(ptr(xf[i], a, 4), ptr(cf, a, 4), alpha, b - a)

    stages = [("reduce", reduce), ("update", update), ("elastic", elastic)]
    if half:
        stages.insert(0, ("pack", pack))

    def run(nthreads, reps):
        pieces = nthreads * 4 if nthreads > 1 else 1
        bounds = np.linspace(0, n, pieces + 1).astype(np.int64)
        spans = [(int(a), int(b)) for a, b in zip(bounds[:-1], bounds[1:]) if b > a]
        times = {}
        with ThreadPoolExecutor(nthreads) as ex:
            for name, fn in stages:
                best = None
                for _ in range(reps):
                    t0 = time.perf_counter()
                    list(ex.map(fn, spans))
                    dt = time.perf_counter() - t0
                    best = dt if best is None else min(best, dt)
                times[name] = best
        return times

    return run(threads, 2), run(1, 1)


def device_facts(torch) -> dict:
    """What the runtime reports about GPU 0, to check the figures the roofline is priced against."""
    p = torch.cuda.get_device_properties(0)
    facts = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2 ** 30, 1)}
    for key, attr, scale in (("arch", "gcnArchName", None), ("l2_cache_MiB", "L2_cache_size", 2 ** 20),
                             ("clock_MHz", "clock_rate", 1000), ("memory_clock_MHz", "memory_clock_rate", 1000),
                             ("memory_bus_bits", "memory_bus_width", 1), ("wavefront", "warp_size", 1)):
        v = getattr(p, attr, None)
        if v is not None:
            facts[key] = v if scale is None else round(v / scale, 1) if scale != 1 else v
    if "memory_clock_MHz" in facts and "memory_bus_bits" in facts:
        # double data rate: two transfers per clock over the whole bus
        facts["memory_GBps_from_clock_and_bus"] = round(2 * facts["memory_clock_MHz"] * 1e6 * facts["memory_bus_bits"] / 8 / 1e9, 1)
    return facts


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--sets", type=int, default=0,
                    help="rotating sets of fresh gradients resident in HBM; 0 = as many as make the rotating "
                         "inputs exceed 1 GB (the caches hold 256 MB), at least 2 and at most 16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="benchmark configuration (3 = the graded one: AlexNet-shaped, k = 8, half-precision transfer)")
    ap.add_argument("--workload", default="alexnet", choices=["alexnet", "vggnet", "googlenet"],
                    help="tensor shapes: AlexNet (the graded workload), the VGGNet parameter count of the paper's "
                         "Table 2, or its GoogLeNet count spread over 128 small tensors")
    ap.add_argument("--chunk", type=int, default=0, help="override elements per chunk")
    ap.add_argument("--blocks-per-cu", type=int, default=-1)
    ap.add_argument("--nontemporal", type=int, default=-1)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the exchange's transfer legs between GPUs are "
              "out of scope); run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_1605_08325_amd as px
    px.load()  # fails loudly if libpxchg.so has not been built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.chunk:
        px.set_option(px.OPT_CHUNK_ELEMS, args.chunk)
    if args.blocks_per_cu >= 0:
        px.set_option(px.OPT_BLOCKS_PER_CU, args.blocks_per_cu)
    if args.nontemporal >= 0:
        px.set_option(px.OPT_NONTEMPORAL, args.nontemporal)

    cfg = wl.config(args.config)
    if args.workload != "alexnet" and args.config != 3:
        print("bench.py: --workload goes with --config 3 only", file=sys.stderr)
        return 2
    counts = {"alexnet": lambda: list(cfg.counts), "vggnet": wl.vggnet_counts,
              "googlenet": lambda: wl.googlenet_scale_counts(cfg.seed)}[args.workload]()
    k, n = cfg.k, sum(counts)
    half = cfg.transfer == "f16"
    wire_t, wire_es, wire_px, wire_name = ((torch.float16, 2, px.F16, "_Float16") if half
                                           else (torch.float32, 4, px.F32, "float"))
    workload_name = cfg.name if args.workload == "alexnet" else f"{args.workload}_sync_k8_f16"
    threads = host_threads()
    table = px.Table(counts)

    # ---- synthetic inputs, resident in HBM before anything is timed
    t_gen = time.perf_counter()
    host_grads0 = None
    grad_sets, pack_sets = [], []
    keep = []
    set_bytes = k * n * (4 + (2 if half else 0))      # one set: k float32 gradients and, if packed, k halves
    n_sets = args.sets if args.sets > 0 else max(2, min(16, -(-10 ** 9 // set_bytes)))
    for s in range(n_sets):
        grads = wl.gaussian_workers(counts, cfg.grad_sigma, cfg.seed, "grad", k, step=s, threads=threads)
        if s == 0:
            host_grads0 = grads
        d_g = [upload(g) for g in grads]
        grad_sets.append([table.bufset(g) for g in d_g])
        if half:
            d_h = [[torch.empty(c, dtype=torch.float16, device="cuda") for c in counts] for _ in range(k)]
            pack_sets.append([table.bufset(h) for h in d_h])
        else:
            pack_sets.append(grad_sets[-1])       # binary32 transfer: the contributions are the gradients themselves
        if s > 0:
            del grads
    w = wl.gaussian_tensors(counts, cfg.param_sigma, cfg.seed, "param")
    v = wl.zeros_tensors(counts)
    d_w, d_v = upload(w), upload(v)
    d_avg = [torch.empty(c, dtype=wire_t, device="cuda") for c in counts]
    s_w, s_v, s_avg = table.bufset(d_w), table.bufset(d_v), table.bufset(d_avg)
    cfg5 = wl.config(5)
    alpha = float(np.float32(0.5 / k))            # configuration 5's rate, 0.5/k
    xs = wl.gaussian_workers(counts, cfg5.param_sigma, cfg5.seed, "worker", k, threads=threads)
    c = wl.gaussian_tensors(counts, cfg5.param_sigma, cfg5.seed, "center")
    d_xs, d_c = [upload(x) for x in xs], upload(c)
    s_xs, s_c = [table.bufset(x) for x in d_xs], table.bufset(d_c)
    orders = wl.worker_orders(cfg5.seed, k, args.steps + args.warmup)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    # the launch stream, looked up once (the binding's default looks it up on every call: 3 us of host time,
    # which shows in the configurations whose kernels take 10..25 us)
    stream = torch.cuda.current_stream().cuda_stream

    def step(i, ev=None, st=stream):
        s = i % len(grad_sets)
        if ev:
            ev[0].record()
        if half:
            px.pack_fp16(table, grad_sets[s], pack_sets[s], stream=st)
        if ev:
            ev[1].record()
        px.reduce_avg(table, pack_sets[s], s_avg, px.AVG, stream=st)
        if ev:
            ev[2].record()
        px.sgd_momentum(table, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=st)
        if ev:
            ev[3].record()
        for j in orders[i]:
            px.easgd(table, s_xs[int(j)], s_c, alpha, stream=st)
        if ev:
            ev[4].record()

    for i in range(args.warmup):
        step(i)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    all_stages = ["pack", "reduce", "update", "elastic"]
    stage_ms = {nm: float(np.mean([events[i][q].elapsed_time(events[i][q + 1]) for i in range(args.steps)]))
                for q, nm in enumerate(all_stages)}
    stage_names = all_stages if half else all_stages[1:]
    # algorithmic bytes per step and per launch
    stage_bytes = {"pack": 6 * k * n, "reduce": (wire_es * k + wire_es) * n, "update": (wire_es + 16) * n,
                   "elastic": 16 * n * k}
    launches = {"pack": 1, "reduce": 1, "update": 1, "elastic": k}
    kernels = {"pack": "pxchg_convert_kernel<float,_Float16>",
               "reduce": f"pxchg_reduce_avg_kernel<{k},{wire_name},{wire_name}>",
               "update": f"pxchg_sgd_momentum_kernel<{wire_name}>", "elastic": "pxchg_easgd_kernel<1>"}
    stages = {}
    for nm in stage_names:
        per_launch_ms = stage_ms[nm] / launches[nm]
        ach = stage_bytes[nm] / launches[nm] / (per_launch_ms * 1e-3) / 1e9
        stages[nm] = {"kernel": kernels[nm], "launches_per_step": launches[nm], "ms_per_launch": round(per_launch_ms, 5),
                      "algorithmic_bytes_per_launch": stage_bytes[nm] // launches[nm], "GBps": round(ach, 1),
                      "frac_of_hbm_peak": round(ach / HBM_PEAK_GBPS, 4),
                      "traffic": MEASURED_TRAFFIC_BYTES.get(nm, (None, None))[0]}
    dominant = max(stage_names, key=lambda nm: stage_ms[nm])
    d = stages[dominant]
    if args.workload != "alexnet" or args.config != 3:
        MEASURED_TRAFFIC_BYTES.clear()  # the counters were collected on configuration 3 only
        for st in stages.values():
            st["traffic"] = None
    traffic = MEASURED_TRAFFIC_BYTES.get(dominant, (None, None))[0]
    roofline = {"bound": "hbm", "kernel": d["kernel"], "achieved": d["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": d["frac_of_hbm_peak"], "traffic": traffic,
                "algorithmic_bytes_per_launch": d["algorithmic_bytes_per_launch"], "ms_per_launch": d["ms_per_launch"]}

    ru_bytes = stage_bytes["reduce"] + stage_bytes["update"]
    ru_ms = stage_ms["reduce"] + stage_ms["update"]
    value = ru_bytes / (ru_ms * 1e-3) / 1e9
    ms_per_step = wall / args.steps * 1e3
    step_bytes = sum(stage_bytes[nm] for nm in stage_names)

    # ---- fused variants (same arithmetic, fewer bytes), timed after the main region
    fused = {}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for i in range(3):
        px.reduce_avg_sgd_momentum(table, pack_sets[0], s_w, s_v, cfg.lr, cfg.mu, cfg.wd, px.AVG, wire_px,
                                   stream=stream)
    ev[0].record()
    for i in range(args.steps):
        px.reduce_avg_sgd_momentum(table, pack_sets[i % len(pack_sets)], s_w, s_v, cfg.lr, cfg.mu, cfg.wd,
                                   px.AVG, wire_px, stream=stream)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fb = (wire_es * k + 16) * n
    fused["reduce_update"] = {"ms": round(ms, 5), "algorithmic_bytes": fb, "GBps": round(fb / ms / 1e6, 1),
                              "frac_of_hbm_peak": round(fb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    for i in range(3):
        px.easgd_round(table, [s_xs[int(j)] for j in orders[i]], s_c, alpha, stream=stream)
    ev[0].record()
    for i in range(args.steps):
        px.easgd_round(table, [s_xs[int(j)] for j in orders[i]], s_c, alpha, stream=stream)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fb = (8 * k + 8) * n
    fused["elastic_round"] = {"ms": round(ms, 5), "algorithmic_bytes": fb, "GBps": round(fb / ms / 1e6, 1),
                              "frac_of_hbm_peak": round(fb / ms / 1e6 / HBM_PEAK_GBPS, 4)}

    # ---- the elastic server's case: nothing but meetings, the center kept in the memory-side cache
    px.set_option(px.OPT_CENTER_RESIDENT, 1)
    try:
        def meetings(i):
            for j in orders[i]:
                px.easgd(table, s_xs[int(j)], s_c, alpha, stream=stream)
        for i in range(3):
            meetings(i)
        ev[0].record()
        for i in range(args.steps):
            meetings(i)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / (args.steps * k)
        fb = 16 * n
        fused["elastic_meeting_center_resident"] = {
            "ms": round(ms, 5), "algorithmic_bytes": fb, "GBps": round(fb / ms / 1e6, 1),
            "note": "PXCHG_OPT_CENTER_RESIDENT=1, meetings back to back: the center's half of the traffic is served "
                    "by the memory-side cache where it fits (256 MB), so this is not an HBM figure"}
        for i in range(3):
            px.easgd_round(table, [s_xs[int(j)] for j in orders[i]], s_c, alpha, stream=stream)
        ev[0].record()
        for i in range(args.steps):
            px.easgd_round(table, [s_xs[int(j)] for j in orders[i]], s_c, alpha, stream=stream)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / args.steps
        fb = (8 * k + 8) * n
        fused["elastic_round_center_resident"] = {"ms": round(ms, 5), "algorithmic_bytes": fb,
                                                  "GBps": round(fb / ms / 1e6, 1)}
    finally:
        px.set_option(px.OPT_CENTER_RESIDENT, 0)

    # ---- diagnostics pass over the averaged gradient (read-only: 2 bytes per element)
    d_stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    for i in range(3):
        px.buffer_stats(table, s_avg, d_stats, stream=stream)
    ev[0].record()
    for i in range(args.steps):
        px.buffer_stats(table, s_avg, d_stats, stream=stream)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fused["diagnostics"] = {"ms": round(ms, 5), "algorithmic_bytes": wire_es * n,
                            "GBps": round(wire_es * n / ms / 1e6, 1),
                            "frac_of_hbm_peak": round(wire_es * n / ms / 1e6 / HBM_PEAK_GBPS, 4),
                            "note": "two launches; an input under 256 MB may sit in the memory-side cache"}

    # ---- the same reduce -> update issued layer by layer (weight and bias of a layer together, last layer
    # first, as back-propagation would hand the gradients over) on two alternating side streams
    per_layer = [table.view(i, min(2, len(counts) - i)) for i in reversed(range(0, len(counts), 2))]
    main_stream = torch.cuda.current_stream()
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    go, done = torch.cuda.Event(), [torch.cuda.Event(), torch.cuda.Event()]

    def per_layer_step():
        go.record(main_stream)
        for st in side:
            st.wait_event(go)
        for li, layer in enumerate(per_layer):          # a view per layer, the whole set's buffer sets
            sp = side[li % 2].cuda_stream
            px.reduce_avg(layer, pack_sets[0], s_avg, px.AVG, stream=sp)
            px.sgd_momentum(layer, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=sp)
        for st, d in zip(side, done):
            d.record(st)
            main_stream.wait_event(d)

    for i in range(3):
        per_layer_step()
    ev[0].record()
    for i in range(args.steps):
        per_layer_step()
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fused["per_layer_two_streams"] = {"ms": round(ms, 5), "algorithmic_bytes": ru_bytes, "layers": len(per_layer),
                                      "launches": 2 * len(per_layer), "GBps": round(ru_bytes / ms / 1e6, 1),
                                      "frac_of_hbm_peak": round(ru_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                                      "note": "reduce+update of the whole set, one view of the table per layer"}

    # ---- one rank's real share of the exchange on a k-GPU node (the transfer legs left out): it packs its own
    # gradient (N elements), sums the k slices of N/k elements it received, and after the second leg updates
    # all N parameters.  The slice is the leading N/k elements of the flat parameter vector.
    share, pieces = n // k, []
    for t_i, cnt in enumerate(counts):
        take = min(cnt, share - sum(p[1] for p in pieces))
        if take <= 0:
            break
        pieces.append((t_i, take))
    slice_table = px.Table([take for _, take in pieces])
    slice_in = [slice_table.bufset([pack_sets[0][i].tensors[t_i][:take] for t_i, take in pieces]) for i in range(k)]
    slice_out = slice_table.bufset([d_avg[t_i][:take] for t_i, take in pieces])
    own_g, own_h = [grad_sets[0][0]], [pack_sets[0][0]]

    def rank_step(e=None):
        if e:
            e[0].record()
        if half:
            px.pack_fp16(table, own_g, own_h, stream=stream)
        if e:
            e[1].record()
        px.reduce_avg(slice_table, slice_in, slice_out, px.AVG, stream=stream)
        if e:
            e[2].record()
        px.sgd_momentum(table, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=stream)
        if e:
            e[3].record()

    for i in range(3):
        rank_step()
    rank_ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for i in range(args.steps):
        rank_step(rank_ev[i])
    torch.cuda.synchronize()
    r_ms = [sum(e[q].elapsed_time(e[q + 1]) for e in rank_ev) / args.steps for q in range(3)]
    r_bytes = [6 * n if half else 0, (wire_es * k + wire_es) * share, (wire_es + 16) * n]
    fused["one_rank_share"] = {
        "ms": round(sum(r_ms), 5), "algorithmic_bytes": sum(r_bytes), "GBps": round(sum(r_bytes) / sum(r_ms) / 1e6, 1),
        "stages_ms": {"pack_own": round(r_ms[0], 5), "reduce_slice": round(r_ms[1], 5), "update_all": round(r_ms[2], 5)},
        "slice_elems": share,
        "note": f"pack of the rank's own gradient, reduce of {k} slices of N/{k} elements, update of all N"}

    # ---- the whole step captured once into a HIP graph and replayed (the calls allocate nothing and record
    # no memset): what is left of a step when the host's per-call cost is gone
    graph = torch.cuda.CUDAGraph()
    cap = torch.cuda.Stream()
    cap.wait_stream(main_stream)
    with torch.cuda.stream(cap):
        with torch.cuda.graph(graph, stream=cap):
            step(0, st=cap.cuda_stream)
    main_stream.wait_stream(cap)
    torch.cuda.synchronize()
    for i in range(3):
        graph.replay()
    ev[0].record()
    for i in range(args.steps):
        graph.replay()
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fused["step_from_hip_graph"] = {"ms": round(ms, 5), "algorithmic_bytes": step_bytes,
                                    "GBps": round(step_bytes / ms / 1e6, 1),
                                    "eager_ms": round(ms_per_step, 5)}

    # ---- a plain copy through the same kernel family (k = 1, no divide: out = in) as a
    # reference for what HBM sustains here, and as the known-size kernel that the
    # hardware-counter readings are scaled by
    d_copy = [torch.empty(c_, dtype=torch.float32, device="cuda") for c_ in counts]
    s_copy = table.bufset(d_copy)
    for i in range(3):
        px.reduce_avg(table, [grad_sets[0][i % k]], s_copy, px.SUM, stream=stream)
    ev[0].record()
    for i in range(args.steps):
        px.reduce_avg(table, [grad_sets[i % len(grad_sets)][i % k]], s_copy, px.SUM, stream=stream)
    ev[1].record()
    torch.cuda.synchronize()
    copy_ms = ev[0].elapsed_time(ev[1]) / args.steps
    copy_gbps = 8 * n / copy_ms / 1e6

    # ---- weight averaging (Section 4's other scheme): the same reduce over the k workers' float32 weights and
    # over their velocities (the float32 gradient buffers stand in for those), one launch each
    for i in range(3):
        px.reduce_avg(table, s_xs, s_copy, px.AVG, stream=stream)
    ev[0].record()
    for i in range(args.steps):
        px.reduce_avg(table, s_xs if i % 2 == 0 else grad_sets[0], s_copy, px.AVG, stream=stream)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / args.steps
    fb = (4 * k + 4) * n
    fused["weight_averaging"] = {"ms": round(ms, 5), "algorithmic_bytes": fb, "GBps": round(fb / ms / 1e6, 1),
                                 "frac_of_hbm_peak": round(fb / ms / 1e6 / HBM_PEAK_GBPS, 4),
                                 "note": f"pxchg_reduce_avg over {k} float32 sets, per launch (weights, then velocities)"}

    # ---- the oracle on the host cores, same workload (a baseline, not a target)
    baseline = None
    if not args.no_cpu_baseline:
        t, t1 = cpu_baseline(counts, host_grads0, w, v, xs, c, [int(j) for j in orders[0]], cfg, alpha, threads)
        cpu_ru = ru_bytes / (t["reduce"] + t["update"]) / 1e9
        baseline = {"value": round(cpu_ru, 2), "unit": "GB/s", "cores": threads, "kind": "oracle",
                    "sample": "the full workload, one step, element range split over the threads, best of 2 "
                              "per stage (same byte accounting as the GPU figure)",
                    "stage_seconds": {kk: round(vv, 4) for kk, vv in t.items()},
                    "step_GBps": round(step_bytes / sum(t.values()) / 1e9, 2),
                    "single_thread": {"value": round(ru_bytes / (t1["reduce"] + t1["update"]) / 1e9, 2),
                                      "stage_seconds": {kk: round(vv, 4) for kk, vv in t1.items()}}}

    out = {
        "metric": "reduce+update GB/s on AlexNet-shaped 61M params, k=8 (fraction of HBM peak)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload_name, "transfer_dtype": cfg.transfer, "n_params": n, "n_tensors": len(counts), "k": k,
                   "step": (f"pack x{k} -> " if half else "") + f"reduce_avg {cfg.transfer}->{cfg.transfer} -> "
                           f"sgd_momentum ({cfg.transfer} grad) -> {k} easgd meetings",
                   "gradient_sets": len(grad_sets), "chunk_elems": px.get_option(px.OPT_CHUNK_ELEMS),
                   "blocks_per_cu": px.get_option(px.OPT_BLOCKS_PER_CU),
                   "nontemporal": px.get_option(px.OPT_NONTEMPORAL),
                   "seed": cfg.seed, "numpy": np.__version__},
        "value_frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "reduce_update_ms": round(ru_ms, 5),
        "step_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "stages": stages,
        "extras": fused,
        "copy_reference": {"what": "plain float32 copy of the same tensor set (pxchg_reduce_avg, k=1, sum), "
                                   "read+write bytes", "kernel": "pxchg_reduce_avg_kernel<1,float,float>",
                           "ms": round(copy_ms, 5), "bytes": 8 * n, "GBps": round(copy_gbps, 1),
                           "frac_of_hbm_peak": round(copy_gbps / HBM_PEAK_GBPS, 4)},
        "cpu_baseline": baseline,
        "setup_seconds": round(t_gen, 1),
        "device": device_facts(torch),
    }
    # the same achieved rates against what a plain copy through the same kernel family sustains on this machine
    out["roofline"]["frac_of_copy_kernel"] = round(out["roofline"]["achieved"] / copy_gbps, 4)
    out["value_frac_of_copy_kernel"] = round(value / copy_gbps, 4)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
