"""Builds libpxchg.so for gfx950 with hipcc, in-tree, next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpxchg.so")
SOURCES = ["pxchg_host.hip", "pxchg_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # every product and sum is rounded on its own: the results are defined that way
    "-ffp-contract=off",
    # no compiler-generated packed-FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


ALL_POLICIES_LIB = os.path.join(ROOT, "tests", "_build", "libpxchg_allpolicies.so")


def build_lib(verbose: bool = False, all_policies: bool = False, out: str = "") -> str:
    """Compile every HIP source and link the shared library.  Always rebuilds.

    The regular library holds each kernel with its own cache policy and with the plain one.  all_policies=True
    makes the tuning build (every kernel with all six policies, -DPXCHG_ALL_POLICIES), which the policy tests
    and A/B measurements load from tests/_build/; it is never the product."""
    out = out or (ALL_POLICIES_LIB if all_policies else LIB)
    os.makedirs(os.path.dirname(out), exist_ok=True)
    tag = ".allpol" if all_policies else ""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(os.path.dirname(out) if all_policies else CSRC, src.replace(".hip", tag + ".o"))
        cmd = [HIPCC, *FLAGS, *(["-DPXCHG_ALL_POLICIES"] if all_policies else []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((subprocess.Popen(cmd), cmd))
        objs.append(obj)
    for p, cmd in procs:
        if p.wait() != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    tmp = out + f".{os.getpid()}.tmp"
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv, all_policies="--all-policies" in sys.argv))
