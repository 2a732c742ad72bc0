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

Two sets of figures per stage.  `ms_per_launch` is the stage inside the step, as
an exchange runs it: the update reads the mean the reduce has just written, the
reduce reads what the pack has just written, and what is left of those in the
256 MB memory-side cache helps.  `cold_ms` is the stage alone in a loop over
rotating operand sets, so that every operand (inputs, outputs, in-place state)
was last touched at least 1 GB of traffic ago: a pure HBM figure.  `value_cold`
is the metric from the cold figures.

`configs` holds every stage (pack where the transfer is half precision, reduce,
update, the elastic meeting) for the other benchmark configurations and the
paper's two other model sizes, each cold (operand sets
rotating over more than 1 GB) and warm (one operand set over and over).

`extras` holds what is measured after the timed region, each over the same number
of repetitions: the fused reduce+update and the fused elastic round (cold), the
elastic kernels with the center kept in the memory-side cache, the diagnostics
pass (warm and cold), the layer-wise exchange on grouped layers, alone and
overlapped with a stand-in gradient producer, one rank's share on an 8-GPU node,
the whole step replayed from a HIP graph, and weight averaging.

`cpu_baseline` is the CPU oracle timed on the host cores on the same workload.
It is a reported baseline (and the only place this program touches the oracle),
never a fallback: without the built HIP library this program fails.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak
COLD_BYTES = 10 ** 9    # an operand counts as cold when this much other traffic has passed since its last use

# HBM traffic per launch is read, at run time, from the committed summary of the hardware-counter runs on this
# same workload: read and write requests between the L2 caches and the memory fabric, counted by size, which
# gives bytes without any scale factor.  (kernel name as the summary prints it, what must also be in the row)
TRAFFIC_PROFILE = os.path.join("profiles", "bench_alexnet_k8_request_sizes_and_utilisation.txt")
TRAFFIC_ROWS = {
    "pack": ("pxchg_convert_kernel<float, _Float16", ""),
    "reduce": ("pxchg_reduce_avg_kernel<8, _Float16, _Float16", ""),
    "update": ("pxchg_sgd_momentum_kernel<_Float16", ""),
    "elastic": ("pxchg_easgd_kernel<1,", "false>"),
    "fused_reduce_update": ("pxchg_reduce_avg_sgd_momentum_kernel<8, _Float16, true", ""),
    "fused_elastic_round": ("pxchg_easgd_kernel<8,", "false>"),
}


def measured_traffic() -> dict:
    """stage -> bytes per launch from the counter summary (64- and 128-byte read requests, 64-byte write
    requests), or {} if the file is not there.  A row ends in: rd64 rd128 readMB algRdMB wr64 writeMB algWrMB ratio."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.search(r"\s(\d+)\s+(\d+)\s+[\d.]+\s+[\d.]+\s+(\d+)\s+[\d.]+\s+[\d.]+\s+[\d.]+\s*$", line)
        if not m:
            continue
        for stage, (prefix, also) in TRAFFIC_ROWS.items():
            if line.startswith(prefix) and also in line.split("[")[0] and stage not in out:
                rd64, rd128, wr64 = (int(g) for g in m.groups())
                out[stage] = rd64 * 64 + rd128 * 128 + wr64 * 64
    return out


def host_threads():
    """(threads the oracle baseline uses, cores this process may run on).  The first is the second unless the
    environment asks for fewer (OMP_NUM_THREADS, which a shared box sets to this job's share)."""
    avail = len(os.sched_getaffinity(0))
    n = avail
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, n), avail


def upload(tensors):
    import torch
    return [torch.from_numpy(np.ascontiguousarray(a)).to("cuda") for a in tensors]


def cpu_baseline(counts, grads, w, v, xs, c, order, cfg, alpha, threads):
    """The oracle, as it stands, on the host cores: same stages, same inputs.  Returns per-stage seconds with
    all `threads` host threads (element range split over them, best of 3) and with one thread."""
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

    return run(threads, 3), run(1, 1)


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


def rate(nbytes, ms):
    gbps = nbytes / ms / 1e6
    return {"ms": round(ms, 5), "algorithmic_bytes": int(nbytes), "GBps": round(gbps, 1),
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}


class Clock:
    """HIP events on torch's current stream, which is the stream every library call below is given."""

    def __init__(self, torch, reps):
        self.torch, self.reps = torch, reps
        self.ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def loop(self, fn, reps=None, warm=3):
        """Mean milliseconds of fn(i) over `reps` calls issued back to back, after `warm` untimed ones."""
        reps = reps or self.reps
        for i in range(warm):
            fn(i)
        self.ev[0].record()
        for i in range(reps):
            fn(warm + i)
        self.ev[1].record()
        self.torch.cuda.synchronize()
        return self.ev[0].elapsed_time(self.ev[1]) / reps


def rotation(per_set_bytes, at_least=2, at_most=64):
    """Number of operand sets to rotate over so that a set comes back only after COLD_BYTES of other traffic."""
    return int(max(at_least, min(at_most, -(-COLD_BYTES // max(1, per_set_bytes)) + 1)))


def bench_config(px, torch, clock, name, counts, k, transfer, lr, mu, wd, alpha, stream, seed, note=None):
    """reduce -> update (and one elastic meeting) on one configuration's shapes: `cold` with every operand set
    rotating over more than COLD_BYTES, `warm` with one operand set over and over (what a loop that does nothing
    else between exchanges would see: small sets then live in the caches).  Inputs are N(0, 0.01^2) draws made on
    the device from the configuration's seed (timing only; the parity tests use the host-drawn inputs)."""
    n = sum(counts)
    half = transfer == "f16"
    wire_t, es = (torch.float16, 2) if half else (torch.float32, 4)
    table = px.Table(counts)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)

    def draw(dtype):
        flat = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0.0, 0.01, generator=gen).to(dtype)
        out, o = [], 0
        for c_ in counts:                       # one allocation per tensor, as the model holds them
            out.append(flat[o:o + c_].clone())
            o += c_
        return out

    set_bytes = n * (k * es + es + 8)           # contributions, mean, parameters and velocity of one operand set
    n_rot = rotation(set_bytes)
    sets, grads = [], []
    for _ in range(n_rot):
        contrib = [table.bufset(draw(wire_t)) for _ in range(k)]
        mean = table.bufset([torch.empty(c_, dtype=wire_t, device="cuda") for c_ in counts])
        sets.append((contrib, mean, table.bufset(draw(torch.float32)), table.bufset(draw(torch.float32))))
        if half:                                # the float32 gradients that the pack turns into the contributions
            grads.append([table.bufset(draw(torch.float32)) for _ in range(k)])
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(clock.reps)]

    def run(rotating):
        def one(i, e=None):
            contrib, mean, w_, v_ = sets[i % n_rot if rotating else 0]
            if e:
                e[0].record()
            px.reduce_avg(table, contrib, mean, px.AVG, stream=stream)
            if e:
                e[1].record()
            px.sgd_momentum(table, mean, w_, v_, lr, mu, wd, stream=stream)
            if e:
                e[2].record()
        for i in range(3):
            one(i)
        for i in range(clock.reps):
            one(3 + i, ev[i])
        torch.cuda.synchronize()
        r_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
        u_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
        return r_ms, u_ms

    r_bytes, u_bytes = (k * es + es) * n, (es + 16) * n
    out = {"n_params": n, "n_tensors": len(counts), "k": k, "transfer": transfer, "operand_sets": n_rot}
    for label, rotating in (("cold", True), ("warm", False)):
        r_ms, u_ms = run(rotating)
        out[label] = {"reduce_ms": round(r_ms, 5), "update_ms": round(u_ms, 5),
                      "reduce_GBps": round(r_bytes / r_ms / 1e6, 1), "update_GBps": round(u_bytes / u_ms / 1e6, 1),
                      "reduce_update_GBps": round((r_bytes + u_bytes) / (r_ms + u_ms) / 1e6, 1),
                      "frac_of_hbm_peak": round((r_bytes + u_bytes) / (r_ms + u_ms) / 1e6 / HBM_PEAK_GBPS, 4)}
    if half:
        for label, rotating in (("cold", True), ("warm", False)):
            ms = clock.loop(lambda i: px.pack_fp16(table, grads[i % n_rot if rotating else 0],
                                                   sets[i % n_rot if rotating else 0][0], stream=stream))
            out[label]["pack_ms"] = round(ms, 5)
            out[label]["pack_GBps"] = round(6 * k * n / ms / 1e6, 1)
    if alpha:
        # the elastic meeting: parameters of one set meet the velocity buffer of the next as "center"
        def meet(i, rotating=True):
            a, b = (i % n_rot, (i + 1) % n_rot) if rotating else (0, 0)
            px.easgd(table, sets[a][2], sets[b][3], alpha, stream=stream)
        for label, rotating in (("cold", True), ("warm", False)):
            ms = clock.loop(lambda i: meet(i, rotating))
            out[label]["meeting_ms"] = round(ms, 5)
            out[label]["meeting_GBps"] = round(16 * n / ms / 1e6, 1)
    if note:
        out["note"] = note
    del sets, grads
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--sets", type=int, default=0,
                    help="rotating sets of fresh gradients resident in HBM; 0 = as many as make the rotating "
                         "inputs exceed 1 GB (the caches hold 256 MB), at least 2 and at most 16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="leave out the other configurations and model sizes")
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="benchmark configuration of the timed step (3 = the graded one: AlexNet-shaped, k = 8, "
                         "half-precision transfer)")
    ap.add_argument("--workload", default="alexnet", choices=["alexnet", "vggnet", "googlenet"],
                    help="tensor shapes: AlexNet (the graded workload), the VGGNet parameter count of the paper's "
                         "Table 2, or its GoogLeNet count spread over 128 small tensors")
    ap.add_argument("--chunk", type=int, default=0, help="override elements per chunk")
    ap.add_argument("--blocks-per-cu", type=int, default=-1)
    ap.add_argument("--tuning-build", action="store_true",
                    help="load the build of the library that holds every cache policy (tests/_build/), for --nontemporal")
    ap.add_argument("--nontemporal", type=int, default=-1)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the exchange's transfer legs between GPUs are "
              "out of scope); run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_1605_08325_amd as px
    if args.tuning_build:
        from paper_1605_08325_amd import build as px_build
        px.binding._lib = px.open_library(px_build.ALL_POLICIES_LIB)
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
    graded = args.workload == "alexnet" and args.config == 3
    counts = {"alexnet": lambda: list(cfg.counts), "vggnet": wl.vggnet_counts,
              "googlenet": lambda: wl.googlenet_scale_counts(cfg.seed)}[args.workload]()
    k, n = cfg.k, sum(counts)
    half = cfg.transfer == "f16"
    wire_t, wire_es, wire_px, wire_name = ((torch.float16, 2, px.F16, "_Float16") if half
                                           else (torch.float32, 4, px.F32, "float"))
    workload_name = cfg.name if args.workload == "alexnet" else f"{args.workload}_sync_k8_f16"
    threads, cores_available = host_threads()
    table = px.Table(counts)
    reps = args.steps

    # ---- synthetic inputs, resident in HBM before anything is timed
    t_gen = time.perf_counter()
    host_grads0 = None
    grad_sets, pack_sets = [], []
    set_bytes = k * n * (4 + (2 if half else 0))      # one set: k float32 gradients and, if packed, k halves
    n_sets = args.sets if args.sets > 0 else max(2, min(16, -(-COLD_BYTES // set_bytes)))
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
    # operand sets for the cold figures: state and outputs rotate too (copies of the same values)
    n_rot = rotation((wire_es + 8) * n, at_least=3)
    rot_state = [(s_w, s_v, s_avg, s_c)]
    for _ in range(n_rot - 1):
        rot_state.append((table.bufset([t.clone() for t in d_w]), table.bufset([t.clone() for t in d_v]),
                          table.bufset([torch.empty_like(t) for t in d_avg]), table.bufset([t.clone() for t in d_c])))
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    # the launch stream, looked up once (the binding's default looks it up on every call: 3 us of host time,
    # which shows in the configurations whose kernels take 10..25 us)
    stream = torch.cuda.current_stream().cuda_stream
    clock = Clock(torch, reps)

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

    # ---- every stage alone, cold: all of its operands rotate, so nothing it touches is still in a cache
    for sw_, sv_, sa_, _ in rot_state[1:]:       # give every mean buffer real contents
        px.reduce_avg(table, pack_sets[0], sa_, px.AVG, stream=stream)
    cold_ms = {}
    if half:
        cold_ms["pack"] = clock.loop(lambda i: px.pack_fp16(table, grad_sets[i % n_sets], pack_sets[i % n_sets], stream=stream))
    cold_ms["reduce"] = clock.loop(lambda i: px.reduce_avg(table, pack_sets[i % n_sets], rot_state[i % n_rot][2], px.AVG,
                                                           stream=stream))
    cold_ms["update"] = clock.loop(lambda i: px.sgd_momentum(table, rot_state[i % n_rot][2], rot_state[i % n_rot][0],
                                                             rot_state[i % n_rot][1], cfg.lr, cfg.mu, cfg.wd, stream=stream))
    cold_ms["elastic"] = clock.loop(lambda i: px.easgd(table, s_xs[i % k], rot_state[i % n_rot][3], alpha, stream=stream)) * k

    # algorithmic bytes per step and per launch
    stage_bytes = {"pack": 6 * k * n, "reduce": (wire_es * k + wire_es) * n, "update": (wire_es + 16) * n,
                   "elastic": 16 * n * k}
    launches = {"pack": 1, "reduce": 1, "update": 1, "elastic": k}
    kernels = {"pack": "pxchg_convert_kernel<float,_Float16>",
               "reduce": f"pxchg_reduce_avg_kernel<{k},{wire_name},{wire_name}>",
               "update": f"pxchg_sgd_momentum_kernel<{wire_name}>", "elastic": "pxchg_easgd_kernel<1>"}
    traffic = measured_traffic() if graded and args.chunk == 0 and args.nontemporal < 0 else {}
    stages = {}
    for nm in stage_names:
        per_launch_ms = stage_ms[nm] / launches[nm]
        per_launch_bytes = stage_bytes[nm] // launches[nm]
        ach = per_launch_bytes / (per_launch_ms * 1e-3) / 1e9
        cold = per_launch_bytes / (cold_ms[nm] / launches[nm] * 1e-3) / 1e9
        stages[nm] = {"kernel": kernels[nm], "launches_per_step": launches[nm], "ms_per_launch": round(per_launch_ms, 5),
                      "algorithmic_bytes_per_launch": per_launch_bytes, "GBps": round(ach, 1),
                      "frac_of_hbm_peak": round(ach / HBM_PEAK_GBPS, 4),
                      "cold_ms": round(cold_ms[nm] / launches[nm], 5), "cold_GBps": round(cold, 1),
                      "cold_frac_of_hbm_peak": round(cold / HBM_PEAK_GBPS, 4),
                      "traffic": traffic.get(nm)}
    dominant = max(stage_names, key=lambda nm: stage_ms[nm])
    d = stages[dominant]
    roofline = {"bound": "hbm", "kernel": d["kernel"], "achieved": d["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": d["frac_of_hbm_peak"], "traffic": d["traffic"],
                "traffic_source": (TRAFFIC_PROFILE + " (64- and 128-byte read requests and 64-byte write requests "
                                   "between L2 and fabric, per launch; a separate counter run of this command)")
                if d["traffic"] else None,
                "algorithmic_bytes_per_launch": d["algorithmic_bytes_per_launch"], "ms_per_launch": d["ms_per_launch"],
                "cold_achieved": d["cold_GBps"], "cold_frac": d["cold_frac_of_hbm_peak"], "cold_ms_per_launch": d["cold_ms"]}

    ru_bytes = stage_bytes["reduce"] + stage_bytes["update"]
    ru_ms = stage_ms["reduce"] + stage_ms["update"]
    value = ru_bytes / (ru_ms * 1e-3) / 1e9
    ru_cold_ms = cold_ms["reduce"] + cold_ms["update"]
    value_cold = ru_bytes / (ru_cold_ms * 1e-3) / 1e9
    ms_per_step = wall / args.steps * 1e3
    step_bytes = sum(stage_bytes[nm] for nm in stage_names)

    # ---- fused variants (same arithmetic, fewer bytes), timed after the main region; cold like the stages
    extras = {}
    ms = clock.loop(lambda i: px.reduce_avg_sgd_momentum(table, pack_sets[i % n_sets], rot_state[i % n_rot][0],
                                                         rot_state[i % n_rot][1], cfg.lr, cfg.mu, cfg.wd, px.AVG, wire_px,
                                                         stream=stream))
    extras["reduce_update"] = dict(rate((wire_es * k + 16) * n, ms), traffic=traffic.get("fused_reduce_update"),
                                   note="pxchg_reduce_avg_sgd_momentum, one launch, cold operands")
    ms = clock.loop(lambda i: px.easgd_round(table, [s_xs[int(j)] for j in orders[i % len(orders)]], rot_state[i % n_rot][3],
                                             alpha, stream=stream))
    extras["elastic_round"] = dict(rate((8 * k + 8) * n, ms), traffic=traffic.get("fused_elastic_round"),
                                   note=f"pxchg_easgd_round of {k}, one launch, cold operands")

    # ---- the elastic server's case: nothing but meetings, the center kept in the memory-side cache
    px.set_option(px.OPT_CENTER_RESIDENT, 1)
    try:
        def meetings(i):
            for j in orders[i % len(orders)]:
                px.easgd(table, s_xs[int(j)], s_c, alpha, stream=stream)
        ms = clock.loop(meetings) / k
        extras["elastic_meeting_center_resident"] = {
            "ms": round(ms, 5), "algorithmic_bytes": 16 * n, "GBps": round(16 * n / ms / 1e6, 1),
            "note": "PXCHG_OPT_CENTER_RESIDENT=1, meetings back to back: the center's half of the traffic is served "
                    "by the memory-side cache where it fits (256 MB), so this is not an HBM figure"}
        ms = clock.loop(lambda i: px.easgd_round(table, [s_xs[int(j)] for j in orders[i % len(orders)]], s_c, alpha,
                                                 stream=stream))
        extras["elastic_round_center_resident"] = {"ms": round(ms, 5), "algorithmic_bytes": (8 * k + 8) * n,
                                                   "GBps": round((8 * k + 8) * n / ms / 1e6, 1)}
    finally:
        px.set_option(px.OPT_CENTER_RESIDENT, 0)

    # ---- diagnostics pass (read-only: 2 bytes per element): on the mean over and over (it then sits in the
    # memory-side cache), and cold, over the k packed sets in turn
    d_stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    ms = clock.loop(lambda i: px.buffer_stats(table, s_avg, d_stats, stream=stream))
    extras["diagnostics"] = dict(rate(wire_es * n, ms), note="two launches; the same 122 MB input every time, which then "
                                                             "sits in the memory-side cache: not an HBM figure")
    flat_sets = [s for ps in pack_sets for s in ps]
    ms = clock.loop(lambda i: px.buffer_stats(table, flat_sets[i % len(flat_sets)], d_stats, stream=stream))
    extras["diagnostics_cold"] = dict(rate(wire_es * n, ms), note=f"two launches; input rotating over {len(flat_sets)} sets")
    ms = clock.loop(lambda i: px.buffer_stats_static(table, flat_sets[i % len(flat_sets)], d_stats, stream=stream))
    extras["diagnostics_static_scratch_cold"] = dict(rate(wire_es * n, ms), note="pxchg_buffer_stats_static, same input rotation")

    # ---- the same reduce -> update issued on groups of layers (views of at least 8 M elements, formed from the
    # last layer backwards as back-propagation hands gradients over; small layers share a group) on two
    # alternating side streams.  The whole set goes through the same fork and join (one group, one side stream)
    # for comparison, so that the ratio shows what the grouping costs and not what the stream hand-over costs.
    groups = table.bucketed_views(8_000_000)
    main_stream = torch.cuda.current_stream()
    side = [torch.cuda.Stream(), torch.cuda.Stream()]
    go, done = torch.cuda.Event(), [torch.cuda.Event(), torch.cuda.Event()]

    def forked(i, tables, fused):
        go.record(main_stream)
        for st in side:
            st.wait_event(go)
        for gi, grp in enumerate(tables):               # a view per group, the whole set's buffer sets
            sp = side[gi % 2].cuda_stream
            if fused:
                px.reduce_avg_sgd_momentum(grp, pack_sets[i % n_sets], s_w, s_v, cfg.lr, cfg.mu, cfg.wd, px.AVG, wire_px,
                                           stream=sp)
            else:
                px.reduce_avg(grp, pack_sets[i % n_sets], s_avg, px.AVG, stream=sp)
                px.sgd_momentum(grp, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=sp)
        for st, d_ in zip(side, done):
            d_.record(st)
            main_stream.wait_event(d_)

    ms = clock.loop(lambda i: forked(i, groups, False))
    ms_whole = clock.loop(lambda i: forked(i, [table], False))
    ms_f = clock.loop(lambda i: forked(i, groups, True))
    ms_f_whole = clock.loop(lambda i: forked(i, [table], True))
    extras["per_layer_two_streams"] = dict(rate(ru_bytes, ms), groups=len(groups), launches=2 * len(groups),
                                           group_elems=[g.total for g in groups], whole_set_ms=round(ms_whole, 5),
                                           ratio_to_whole_set=round(ms / ms_whole, 4),
                                           fused_ms=round(ms_f, 5), fused_whole_set_ms=round(ms_f_whole, 5),
                                           fused_ratio_to_whole_set=round(ms_f / ms_f_whole, 4),
                                           note="reduce+update of the whole set, one view per group of layers, two side "
                                                "streams; whole_set_ms: the same through the same fork and join as one "
                                                "group; fused_*: pxchg_reduce_avg_sgd_momentum per group (one launch each)")

    # ---- overlap with a gradient producer (the overlap the paper names as future work): a producer stream hands
    # the k workers' gradients over group by group, last layers first (here: the pack of that group, which
    # writes the k binary16 gradient sets), and an exchange stream reduces and updates each group as soon as
    # its event fires.  exposed = what is left of the exchange after the producer's last write.
    if half:
        prod, exch = torch.cuda.Stream(), torch.cuda.Stream()
        ready = [torch.cuda.Event() for _ in groups]
        t_start, t_prod, t_end = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        fin = torch.cuda.Event()

        # a compute-bound stand-in for the back-propagation of one group of layers: a bf16 matrix product through
        # torch (matrix cores, little HBM traffic), sized to take about as long as that group's exchange
        mm_a = torch.randn(4096, 4096, dtype=torch.bfloat16, device="cuda")
        mm_b = torch.randn(4096, 4096, dtype=torch.bfloat16, device="cuda")
        mm_c = torch.empty(4096, 4096, dtype=torch.bfloat16, device="cuda")
        compute = [False]

        def backprop_of_group(st):
            if compute[0]:
                with torch.cuda.stream(st):
                    for _ in range(2):
                        torch.mm(mm_a, mm_b, out=mm_c)

        def overlapped(i, timed=False):
            s = i % n_sets
            go.record(main_stream)
            prod.wait_event(go)
            exch.wait_event(go)
            if timed:
                t_start.record(prod)
            for gi, grp in enumerate(groups):
                backprop_of_group(prod)
                px.pack_fp16(grp, grad_sets[s], pack_sets[s], stream=prod.cuda_stream)
                ready[gi].record(prod)
                exch.wait_event(ready[gi])
                px.reduce_avg(grp, pack_sets[s], s_avg, px.AVG, stream=exch.cuda_stream)
                px.sgd_momentum(grp, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=exch.cuda_stream)
            if timed:
                t_prod.record(prod)
                t_end.record(exch)
            fin.record(exch)
            main_stream.wait_event(fin)
            main_stream.wait_stream(prod)

        def serial(i, timed=False):
            s = i % n_sets
            if timed:
                t_start.record(main_stream)
            for grp in groups:
                backprop_of_group(main_stream)
                px.pack_fp16(grp, grad_sets[s], pack_sets[s], stream=stream)
            if timed:
                t_prod.record(main_stream)
            px.reduce_avg(table, pack_sets[s], s_avg, px.AVG, stream=stream)
            px.sgd_momentum(table, s_avg, s_w, s_v, cfg.lr, cfg.mu, cfg.wd, stream=stream)
            if timed:
                t_end.record(main_stream)

        def timed_runs(fn):
            for i in range(3):
                fn(i)
            total, exposed = [], []
            for i in range(reps):
                fn(3 + i, True)
                torch.cuda.synchronize()
                total.append(t_start.elapsed_time(t_end))
                exposed.append(t_prod.elapsed_time(t_end))
            return float(np.mean(total)), float(np.mean(exposed))

        ov_total, ov_exposed = timed_runs(overlapped)
        se_total, se_exposed = timed_runs(serial)
        extras["overlap_with_producer"] = {
            "groups": len(groups), "producer": "pack of each group on its own stream (an HBM-bound stand-in for "
                                               "back-propagation, so it competes with the exchange for bandwidth; "
                                               "a compute-bound producer would leave more of it to the exchange)",
            "overlapped_total_ms": round(ov_total, 5), "exposed_exchange_ms": round(max(ov_exposed, 0.0), 5),
            "serial_total_ms": round(se_total, 5), "serial_exchange_ms": round(se_exposed, 5),
            "note": "exposed_exchange_ms: from the producer's last write to the end of the last update; "
                    "serial: every group produced first, then one reduce and one update over the whole set"}
        compute[0] = True
        ov_total, ov_exposed = timed_runs(overlapped)
        se_total, se_exposed = timed_runs(serial)
        extras["overlap_with_compute_producer"] = {
            "groups": len(groups), "producer": "per group: two 4096^3 bf16 matrix products through torch (a compute-bound "
                                               "stand-in for that group's back-propagation), then the pack of the group",
            "overlapped_total_ms": round(ov_total, 5), "exposed_exchange_ms": round(max(ov_exposed, 0.0), 5),
            "serial_total_ms": round(se_total, 5), "serial_exchange_ms": round(se_exposed, 5),
            "hidden_ms": round(se_total - ov_total, 5),
            "note": "hidden_ms: serial total minus overlapped total.  On one GPU the two streams share the compute "
                    "units (kernels of both are time-sliced: a matrix product and a reduce+update issued together "
                    "each take twice as long), so the exchange no longer waits at the end (exposed_exchange_ms) "
                    "but the step does not get shorter; what the layer-wise form buys in a multi-GPU exchange is "
                    "that the transfer legs, which run on copy engines and links, can start while back-propagation "
                    "still computes"}
        del mm_a, mm_b, mm_c

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
    rank_ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
    for i in range(reps):
        rank_step(rank_ev[i])
    torch.cuda.synchronize()
    r_ms = [sum(e[q].elapsed_time(e[q + 1]) for e in rank_ev) / reps for q in range(3)]
    r_bytes = [6 * n if half else 0, (wire_es * k + wire_es) * share, (wire_es + 16) * n]
    extras["one_rank_share"] = {
        "ms": round(sum(r_ms), 5), "algorithmic_bytes": sum(r_bytes), "GBps": round(sum(r_bytes) / sum(r_ms) / 1e6, 1),
        "stages_ms": {"pack_own": round(r_ms[0], 5), "reduce_slice": round(r_ms[1], 5), "update_all": round(r_ms[2], 5)},
        "slice_elems": share,
        "note": f"pack of the rank's own gradient, reduce of {k} slices of N/{k} elements, update of all N"}
    del slice_in, slice_out, slice_table

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
    ms = clock.loop(lambda i: graph.replay())
    extras["step_from_hip_graph"] = {"ms": round(ms, 5), "algorithmic_bytes": step_bytes,
                                     "GBps": round(step_bytes / ms / 1e6, 1), "eager_ms": round(ms_per_step, 5)}
    del graph

    # ---- a plain copy through the same kernel family (k = 1, no divide: out = in) as a
    # reference for what HBM sustains here, and as the known-size kernel that counter readings can be checked on
    copies = [table.bufset([torch.empty(c_, dtype=torch.float32, device="cuda") for c_ in counts]) for _ in range(3)]
    sources = [g for gs in grad_sets for g in gs]
    copy_ms = clock.loop(lambda i: px.reduce_avg(table, [sources[i % len(sources)]], copies[i % 3], px.SUM, stream=stream))
    copy_gbps = 8 * n / copy_ms / 1e6

    # ---- weight averaging (Section 4's other scheme): the same reduce over the k workers' float32 weights and
    # over their velocities (the float32 gradient buffers stand in for those), one launch each
    ms = clock.loop(lambda i: px.reduce_avg(table, s_xs if i % 2 == 0 else grad_sets[0], copies[i % 3], px.AVG, stream=stream))
    extras["weight_averaging"] = dict(rate((4 * k + 4) * n, ms),
                                      note=f"pxchg_reduce_avg over {k} float32 sets, per launch (weights, then velocities)")
    del copies

    # ---- the other configurations and model sizes: reduce+update (and the meeting), cold and warm
    configs = None
    if graded and not args.no_configs:
        configs = {}
        c1, c2, c4, c5 = wl.config(1), wl.config(2), wl.config(4), wl.config(5)
        for name, cnts, kk, tr, lr_, mu_, wd_, al_, seed_, note in (
                ("1_tiny_k2_f32", list(c1.counts), c1.k, c1.transfer, c1.lr, c1.mu, c1.wd, 0.0625, c1.seed,
                 "12..21 MB per launch: bound by launch cost (about 4 us of host time per call), and cache-resident when warm"),
                ("2_alexnet_k2_f32", list(c2.counts), c2.k, c2.transfer, c2.lr, c2.mu, c2.wd, 0.0, c2.seed, None),
                ("4_many_small_k8_f16", list(c4.counts), c4.k, c4.transfer, c4.lr, c4.mu, c4.wd, 0.0625, c4.seed,
                 "116 ragged tensors, one launch per stage; 126 MB per launch"),
                ("5_alexnet_easgd_k8_f32", list(c5.counts), c5.k, c5.transfer, c5.lr, c5.mu, c5.wd, c5.alpha, c5.seed,
                 "the meeting is this configuration's own step; reduce+update on its float32 buffers is weight averaging plus update"),
                ("googlenet_count_k8_f16", wl.googlenet_scale_counts(c4.seed), 8, "f16", 0.01, 0.9, 0.0, 0.0625, c4.seed + 100,
                 "Table 2's GoogLeNet count (13,378,280) over 128 ragged tensors"),
                ("vggnet_k8_f16", wl.vggnet_counts(), 8, "f16", 0.01, 0.9, 0.0, 0.0625, c5.seed + 100,
                 "Table 2's VGGNet count (138,357,544), 32 tensors")):
            configs[name] = bench_config(px, torch, clock, name, cnts, kk, tr, lr_, mu_, wd_, al_, stream, seed_, note)

    # ---- the oracle on the host cores, same workload (a baseline, not a target)
    baseline = None
    if not args.no_cpu_baseline:
        t, t1 = cpu_baseline(counts, host_grads0, w, v, xs, c, [int(j) for j in orders[0]], cfg, alpha, threads)
        cpu_ru = ru_bytes / (t["reduce"] + t["update"]) / 1e9
        baseline = {"value": round(cpu_ru, 2), "unit": "GB/s", "cores": threads, "cores_available": cores_available,
                    "kind": "oracle",
                    "sample": "the full workload, one step, element range split over the threads, best of 3 "
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
                   "gradient_sets": len(grad_sets), "state_sets_for_cold_figures": n_rot,
                   "chunk_elems": px.get_option(px.OPT_CHUNK_ELEMS),
                   "blocks_per_cu": px.get_option(px.OPT_BLOCKS_PER_CU),
                   "nontemporal": px.get_option(px.OPT_NONTEMPORAL),
                   "seed": cfg.seed, "numpy": np.__version__},
        "value_frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "value_cold": round(value_cold, 1),
        "value_cold_frac_of_hbm_peak": round(value_cold / HBM_PEAK_GBPS, 4),
        "value_note": "value: reduce and update inside the step, as an exchange runs them (the update reads the mean the "
                      "reduce has just written, partly from the memory-side cache); value_cold: each of the two alone, "
                      "every operand rotating out of the caches",
        "reduce_update_ms": round(ru_ms, 5),
        "reduce_update_cold_ms": round(ru_cold_ms, 5),
        "step_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "stages": stages,
        "extras": extras,
        "configs": configs,
        "copy_reference": {"what": "plain float32 copy of the same tensor set (pxchg_reduce_avg, k=1, sum), "
                                   "read+write bytes, cold operands", "kernel": "pxchg_reduce_avg_kernel<1,float,float>",
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
