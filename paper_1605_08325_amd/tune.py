"""A/B measurement of the kernels' tuning choices on one MI355X, all inside one process on one box.

Boxes differ by several percent for the same binary, so a choice (lane layout, idle wavefronts, store policy,
workgroups per chunk) is only ever compared with its alternatives in alternating rounds of one run.  This tool

    python -m paper_1605_08325_amd.tune --build          (on a machine with hipcc; no GPU needed)

compiles the library once per alternative (the kernels' source has `PXCHG_TUNE_*` hooks for exactly these) into
paper_1605_08325_amd/_build/tune/<name>/libpxchg.so, and

    python -m paper_1605_08325_amd.tune --run [--policies | --launch-shapes] [--shape alexnet|small|vggnet|googlenet]

first checks that every alternative produces the same bits as the shipped shape on the same inputs, then times
the exchange calls for each in alternating rounds and prints the medians and the spread: `cold` with every operand
rotating over more than 1 GB (a pure HBM figure), `in step` for reduce -> update back to back on one operand
set (what the benchmark's step does).  --policies does the same for the six cache policies with the tuning
build of the library (tests/_build/libpxchg_allpolicies.so), --launch-shapes for the regular library under other
chunk sizes and persistent grids (PXCHG_OPT_CHUNK_ELEMS, PXCHG_OPT_BLOCKS_PER_CU).  Inputs are N(0, 0.01^2) draws made on the device
from a fixed seed, AlexNet-shaped (61 M parameters, 16 tensors, k = 8), the 116-tensor set of 7 M, VGGNet-shaped
(138 M) or the GoogLeNet count (13.4 M in 128 tensors).
The summaries under profiles/ that justify the shipped choices are this tool's output.
"""
from __future__ import annotations

import argparse
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TUNE_DIR = os.path.join(HERE, "_build", "tune")

# name -> extra compiler flags; "shipped" is the library as it is built for use
VARIANTS = {
    "shipped": [],
    "no_idle_wavefronts": ["-DPXCHG_TUNE_NO_IDLE"],
    "update_1_idle_wavefront": ["-DPXCHG_TUNE_UPDATE_THREADS=192"],
    "update_4_idle_wavefronts": ["-DPXCHG_TUNE_UPDATE_THREADS=384"],
    "meeting_1_idle_wavefront": ["-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    "meeting_3_idle_wavefronts": ["-DPXCHG_TUNE_ELASTIC1_PAD=4"],
    "meeting_5_idle_wavefronts": ["-DPXCHG_TUNE_ELASTIC1_PAD=6"],
    "idle_wavefronts_leave_at_entry": ["-DPXCHG_TUNE_IDLE_EXIT=1"],
    "idle_wavefronts_leave_after_descriptor": ["-DPXCHG_TUNE_IDLE_EXIT=2"],
    "reduce16_no_idle_wavefronts": ["-DPXCHG_TUNE_REDUCE16_IDLE=0"],
    "reduce16_1_idle_wavefront": ["-DPXCHG_TUNE_REDUCE16_IDLE=1"],
    "reduce16_2_idle_wavefronts": ["-DPXCHG_TUNE_REDUCE16_IDLE=2"],
    "reduce16_3_idle_wavefronts": ["-DPXCHG_TUNE_REDUCE16_IDLE=3"],
    "fused_no_idle_wavefront": ["-DPXCHG_TUNE_FUSED_IDLE=0"],
    "fused_1_idle_wavefront": ["-DPXCHG_TUNE_FUSED_IDLE=1"],
    "fused_2_idle_wavefronts": ["-DPXCHG_TUNE_FUSED_IDLE=2"],
    "round8_4_idle_wavefronts": ["-DPXCHG_TUNE_ELASTIC8_PAD=2"],
    "reduce_pointers_by_scalar_loads": ["-DPXCHG_TUNE_REDUCE_POINTERS=0"],
    "reduce_pointers_lane_parallel": ["-DPXCHG_TUNE_REDUCE_POINTERS=1"],
    "pack_128_lanes": ["-DPXCHG_TUNE_CONVERT_LANES=128"],
    "pack_2_parts": ["-DPXCHG_TUNE_CONVERT_PARTS=2"],
    "reduce16_64_lanes": ["-DPXCHG_TUNE_REDUCE16_LANES=64", "-DPXCHG_TUNE_REDUCE16_IDLE=0"],
    "fused_one_part_256_lanes": ["-DPXCHG_TUNE_FUSED_PARTS=1"],
    "fused_one_part_64_lanes_split": ["-DPXCHG_TUNE_FUSED_PARTS=1", "-DPXCHG_TUNE_FUSED_LANES=64"],
    "fused_one_part_128_lanes": ["-DPXCHG_TUNE_FUSED_PARTS=1", "-DPXCHG_TUNE_FUSED_LANES=128"],
    "meeting_one_part_128_lanes": ["-DPXCHG_TUNE_ELASTIC1_PARTS=1", "-DPXCHG_TUNE_ELASTIC1_LANES=128", "-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    "meeting_one_part_64_lanes": ["-DPXCHG_TUNE_ELASTIC1_PARTS=1", "-DPXCHG_TUNE_ELASTIC1_LANES=64", "-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    "meeting_one_part_256_lanes": ["-DPXCHG_TUNE_ELASTIC1_PARTS=1", "-DPXCHG_TUNE_ELASTIC1_LANES=256", "-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    "meeting_2_parts_128_lanes": ["-DPXCHG_TUNE_ELASTIC1_PARTS=2", "-DPXCHG_TUNE_ELASTIC1_LANES=128", "-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    "meeting_4_parts_64_lanes": ["-DPXCHG_TUNE_ELASTIC1_PARTS=4", "-DPXCHG_TUNE_ELASTIC1_LANES=64", "-DPXCHG_TUNE_ELASTIC1_PAD=2"],
    # two workgroups per chunk for the kernels that ship with one
    "update_2_parts": ["-DPXCHG_TUNE_UPDATE_PARTS=2"],
    "update_2_parts_no_idle": ["-DPXCHG_TUNE_UPDATE_PARTS=2", "-DPXCHG_TUNE_NO_IDLE"],
    "reduce16_2_parts": ["-DPXCHG_TUNE_REDUCE16_PARTS=2", "-DPXCHG_TUNE_REDUCE16_IDLE=0"],
    "reduce16_256_lanes": ["-DPXCHG_TUNE_REDUCE16_LANES=256", "-DPXCHG_TUNE_REDUCE16_IDLE=0"],
    "round8_4_parts_128_lanes": ["-DPXCHG_TUNE_ELASTIC8_PARTS=4"],
    "round8_one_part_512_lanes": ["-DPXCHG_TUNE_ELASTIC8_PARTS=1"],
    "round8_one_part_256_lanes": ["-DPXCHG_TUNE_ELASTIC8_PARTS=1", "-DPXCHG_TUNE_ELASTIC8_LANES=256"],
    "round8_one_part_128_lanes": ["-DPXCHG_TUNE_ELASTIC8_PARTS=1", "-DPXCHG_TUNE_ELASTIC8_LANES=128"],
    "reduce_policy_3": ["-DPXCHG_TUNE_REDUCE_POLICY=3"],
    "reduce_policy_4": ["-DPXCHG_TUNE_REDUCE_POLICY=4"],
    # block shapes of the diagnostics (they are part of that call's definition: the sum's bits differ, by design)
    "diagnostics_4_waves_64_chunks": ["-DPXCHG_STATS_BLOCK_CHUNKS=64"],
    "diagnostics_8_waves_64_chunks": ["-DPXCHG_STATS_WAVES=8", "-DPXCHG_STATS_BLOCK_CHUNKS=64"],
    "diagnostics_16_waves_256_chunks": ["-DPXCHG_STATS_WAVES=16", "-DPXCHG_STATS_BLOCK_CHUNKS=256"],
}


def build_variants(names=None) -> None:
    from paper_1605_08325_amd import build as b
    names = list(names or VARIANTS)

    def one(name):
        d = os.path.join(TUNE_DIR, name)
        os.makedirs(d, exist_ok=True)
        objs = []
        for src in b.SOURCES:
            obj = os.path.join(d, src.replace(".hip", ".o"))
            subprocess.run([b.HIPCC, *b.FLAGS, *VARIANTS[name], "-c", os.path.join(b.CSRC, src), "-o", obj],
                           check=True, stderr=subprocess.DEVNULL)
            objs.append(obj)
        subprocess.run([b.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", os.path.join(d, "libpxchg.so")],
                       check=True)
        for o in objs:
            os.remove(o)
        return name

    with ThreadPoolExecutor(4) as ex:
        for name in ex.map(one, names):
            print("built", name, flush=True)


def run(args) -> int:
    import numpy as np
    import torch

    import paper_1605_08325_amd as px
    import workloads as wl

    torch.cuda.set_device(0)
    counts = {"alexnet": wl.alexnet_counts, "small": lambda: list(wl.config(4).counts), "vggnet": wl.vggnet_counts,
              "googlenet": lambda: wl.googlenet_scale_counts(wl.config(4).seed)}[args.shape]()
    n, k = sum(counts), 8
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20160526)

    def draw(dtype):
        flat = torch.empty(n, dtype=torch.float32, device="cuda").normal_(0, 0.01, generator=gen).to(dtype)
        out, o = [], 0
        for c in counts:
            out.append(flat[o:o + c].clone())
            o += c
        return out

    big = n > 30_000_000
    n_in, n_state = (2, 3) if big else (10, 24)     # operand sets to rotate over: more than 1 GB between two uses
    halves = [[draw(torch.float16) for _ in range(k)] for _ in range(n_in)]
    packed = [[[torch.empty_like(t) for t in ts] for ts in s] for s in halves] if big else None    # the pack's output
    floats = [draw(torch.float32) for _ in range(k)]
    state = [(draw(torch.float32), draw(torch.float32), draw(torch.float16), draw(torch.float32)) for _ in range(n_state)]
    pristine = [[t.clone() for t in ts] for ts in (*state[0], *floats)]
    stream = torch.cuda.current_stream().cuda_stream
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

    def loop(fn, warm=3):
        for i in range(warm):
            fn(i)
        ev[0].record()
        for i in range(args.reps):
            fn(warm + i)
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / args.reps * 1e3

    shapes = {}
    if args.launch_shapes:
        # the regular library under other launch shapes: elements per chunk, persistent workgroups per compute unit
        shapes = {f"chunk {c:5d}, {w:2d} wg/CU" if w else f"chunk {c:5d}, one wg per chunk": (c, w)
                  for c, w in ((512, 0), (1024, 0), (2048, 0), (512, 8), (512, 16), (512, 32), (1024, 8), (2048, 4), (4096, 4))}
        libs = {nm: (px.library_path(), -1) for nm in shapes}
    elif args.policies:
        from paper_1605_08325_amd import build as b
        libs = {f"policy {p}" if p >= 0 else "own policy": (b.ALL_POLICIES_LIB, p) for p in (-1, 0, 1, 2, 3, 4, 5)}
    else:
        names = args.variants.split(",") if args.variants else list(VARIANTS)
        libs = {nm: (os.path.join(TUNE_DIR, nm, "libpxchg.so"), -1) for nm in names}
    opened = {}
    results, reference = {}, None
    columns = ["pack", "reduce", "update", "meeting", "fused r+u", "round of 8", "diagnostics", "in-step reduce",
               "in-step update"]
    d_stats = torch.zeros(3, dtype=torch.int64, device="cuda")
    for rnd in range(args.rounds):
        for nm, (path, policy) in libs.items():
            lib = opened.setdefault(path, px.open_library(path))
            with px.using(lib):
                px.set_option(px.OPT_NONTEMPORAL, policy)
                if nm in shapes:
                    px.set_option(px.OPT_CHUNK_ELEMS, shapes[nm][0])
                    px.set_option(px.OPT_BLOCKS_PER_CU, shapes[nm][1])
                table = px.Table(counts)
                hs = [[table.bufset(t) for t in s] for s in halves]
                ps = [[table.bufset(t) for t in s] for s in packed] if big else None
                fs = [table.bufset(t) for t in floats]
                st = [tuple(table.bufset(t) for t in s) for s in state]
                if rnd == 0:
                    # same bits as the first alternative, on private copies of the same inputs
                    w0, v0, m0, c0, *x0 = [[t.clone() for t in ts] for ts in pristine]
                    sw, sv, sm, sc = (table.bufset(t) for t in (w0, v0, m0, c0))
                    sx = [table.bufset(t) for t in x0]
                    px.reduce_avg(table, hs[0], sm, px.AVG)
                    px.sgd_momentum(table, sm, sw, sv, 0.01, 0.9, 5e-4)
                    px.reduce_avg_sgd_momentum(table, hs[1 % n_in], sw, sv, 0.01, 0.9, 5e-4, px.AVG, px.F16)
                    px.easgd(table, sx[0], sc, 0.0625)
                    px.easgd_round(table, sx, sc, 0.0625)
                    torch.cuda.synchronize()
                    got = [w0, v0, m0, c0, x0[0], x0[k - 1]]
                    if reference is None:
                        reference = [[t.clone() for t in ts] for ts in got]
                    else:
                        for a, b_ in zip(reference, got):
                            for ta, tb in zip(a, b_):
                                if not torch.equal(ta, tb):
                                    print(f"{nm}: results differ from {next(iter(libs))}", file=sys.stderr)
                                    return 1
                    del sw, sv, sm, sc, sx
                row = [
                    loop(lambda i: px.pack_fp16(table, fs, ps[i % n_in], stream=stream)) if big else float("nan"),
                    loop(lambda i: px.reduce_avg(table, hs[i % n_in], st[i % n_state][2], px.AVG, stream=stream)),
                    loop(lambda i: px.sgd_momentum(table, st[i % n_state][2], st[i % n_state][0], st[i % n_state][1], 0.01, 0.9,
                                                   0.0, stream=stream)),
                    loop(lambda i: px.easgd(table, fs[i % k], st[i % n_state][3], 0.0625, stream=stream)),
                    loop(lambda i: px.reduce_avg_sgd_momentum(table, hs[i % n_in], st[i % n_state][0], st[i % n_state][1], 0.01,
                                                              0.9, 0.0, px.AVG, px.F16, stream=stream)),
                    loop(lambda i: px.easgd_round(table, fs, st[i % n_state][3], 0.0625, stream=stream)),
                    loop(lambda i: px.buffer_stats(table, hs[i % n_in][i % k], d_stats, stream=stream)),
                ]
                # reduce -> update back to back on one state set, as the benchmark's step runs them
                acc = [0.0, 0.0]
                for i in range(3 + args.reps):
                    ev[0].record()
                    px.reduce_avg(table, hs[i % n_in], st[0][2], px.AVG, stream=stream)
                    ev[1].record()
                    px.sgd_momentum(table, st[0][2], st[0][0], st[0][1], 0.01, 0.9, 0.0, stream=stream)
                    ev[2].record()
                    torch.cuda.synchronize()
                    if i >= 3:
                        acc[0] += ev[0].elapsed_time(ev[1])
                        acc[1] += ev[1].elapsed_time(ev[2])
                row += [acc[0] / args.reps * 1e3, acc[1] / args.reps * 1e3]
                results.setdefault(nm, []).append(row)
                px.set_option(px.OPT_NONTEMPORAL, -1)
                px.set_option(px.OPT_CHUNK_ELEMS, 512)
                px.set_option(px.OPT_BLOCKS_PER_CU, 0)
                del hs, ps, fs, st, table
        print(f"round {rnd + 1} of {args.rounds} done", flush=True)

    print(f"\n{args.shape}: {n} parameters in {len(counts)} tensors, k = {k}; microseconds per launch, median of "
          f"{args.rounds} alternating rounds of {args.reps} launches (largest deviation of a round from the median in "
          f"brackets, over all columns); every alternative gave the same bits")
    print(f"{'alternative':28s} " + " ".join(f"{c:>14s}" for c in columns))
    for nm, rows in results.items():
        a = np.array(rows)
        med = np.nanmedian(a, axis=0)
        dev = np.nanmax(np.abs(a - med) / med) * 100
        print(f"{nm:28s} " + " ".join(f"{m:14.1f}" for m in med) + f"   [{dev:.1f} %]")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--build", action="store_true", help="compile the alternatives (hipcc; no GPU needed)")
    ap.add_argument("--run", action="store_true", help="check and time them on the GPU")
    ap.add_argument("--policies", action="store_true", help="time the six cache policies of the tuning build instead")
    ap.add_argument("--launch-shapes", action="store_true",
                    help="time the regular library under other chunk sizes and persistent grids instead")
    ap.add_argument("--variants", default="", help="comma-separated subset of: " + ", ".join(VARIANTS))
    ap.add_argument("--shape", default="alexnet", choices=["alexnet", "small", "vggnet", "googlenet"])
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--reps", type=int, default=30)
    args = ap.parse_args()
    if args.build:
        build_variants(args.variants.split(",") if args.variants else None)
    if args.run:
        return run(args)
    if not args.build:
        ap.print_help()
    return 0


if __name__ == "__main__":
    sys.exit(main())
