"""Python face of the CPU oracle (test infrastructure, never the product path).

Thin ctypes marshalling over ``pxchg_oracle.c``: the arithmetic lives in the C
file, one scalar loop per step of the exchange (Sections 3.2 and 4 of the
paper).  Only tests, the smoke check and the benchmark's CPU-baseline leg may
import this package; it imports nothing from the HIP library or its binding.

Multi-tensor calls are a Python loop over tensors calling the flat C function:
there is no blocking, fusion or reordering here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pxchg_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libpxchg_oracle.so")

F32, F16 = 0, 1
AVG, SUM = 0, 1

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
          "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the path of the shared object."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    os.makedirs(os.path.dirname(_LIB), exist_ok=True)
    tmp = _LIB + f".{os.getpid()}.tmp"
    subprocess.run(["gcc", *CFLAGS, _SRC, "-o", tmp], check=True)
    os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # PXCHG_ORACLE_LIB: a prebuilt oracle to load instead (the mutation test points it at deliberately
        # broken builds to show that the pins notice)
        L = ctypes.CDLL(os.environ.get("PXCHG_ORACLE_LIB") or build())
        i64, vp, f = ctypes.c_int64, ctypes.c_void_p, ctypes.c_float
        L.oracle_f32_to_f16_bits.argtypes = [ctypes.c_uint32]
        L.oracle_f32_to_f16_bits.restype = ctypes.c_uint16
        L.oracle_f16_to_f32_bits.argtypes = [ctypes.c_uint16]
        L.oracle_f16_to_f32_bits.restype = ctypes.c_uint32
        L.oracle_pack_fp16.argtypes = [vp, vp, i64]
        L.oracle_pack_fp16.restype = None
        L.oracle_unpack_fp16.argtypes = [vp, vp, i64]
        L.oracle_unpack_fp16.restype = None
        L.oracle_reduce_avg.argtypes = [ctypes.c_int, ctypes.POINTER(vp), ctypes.c_int,
                                        vp, ctypes.c_int, ctypes.c_int, i64]
        L.oracle_reduce_avg.restype = ctypes.c_int
        L.oracle_sgd_momentum.argtypes = [vp, ctypes.c_int, vp, vp, f, f, f, i64]
        L.oracle_sgd_momentum.restype = ctypes.c_int
        L.oracle_easgd.argtypes = [vp, vp, f, i64]
        L.oracle_easgd.restype = ctypes.c_int
        L.oracle_stats.argtypes = [vp, ctypes.c_int, i64, ctypes.POINTER(ctypes.c_uint64),
                                   ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
        L.oracle_stats.restype = ctypes.c_int
        L.oracle_stats_ordered.argtypes = [ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(i64), ctypes.c_int, i64,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_uint64),
                                           ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
        L.oracle_stats_ordered.restype = ctypes.c_int
        _lib = L
    return _lib


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    if not isinstance(a, np.ndarray) or a.dtype != dtype or a.ndim != 1 \
            or not a.flags.c_contiguous:
        raise TypeError(f"expected contiguous 1-D {np.dtype(dtype)} array")
    return a


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError("float32 or float16 expected")


# -- scalar conversions ---------------------------------------------------------

def f32_to_f16_bits(x: int) -> int:
    return int(lib().oracle_f32_to_f16_bits(x & 0xFFFFFFFF))


def f16_to_f32_bits(h: int) -> int:
    return int(lib().oracle_f16_to_f32_bits(h & 0xFFFF))


# -- flat (one tensor) ------------------------------------------------------------

def pack_fp16(g: np.ndarray) -> np.ndarray:
    _chk(g, np.float32)
    h = np.empty(g.shape, np.float16)
    lib().oracle_pack_fp16(g.ctypes.data, h.ctypes.data, g.size)
    return h


def unpack_fp16(h: np.ndarray) -> np.ndarray:
    _chk(h, np.float16)
    g = np.empty(h.shape, np.float32)
    lib().oracle_unpack_fp16(h.ctypes.data, g.ctypes.data, h.size)
    return g


def reduce_avg(contrib: Sequence[np.ndarray], out_dtype=np.float32, mode: int = AVG) -> np.ndarray:
    k = len(contrib)
    if k < 1:
        raise ValueError("k >= 1")
    dt = contrib[0].dtype
    n = contrib[0].size
    for c in contrib:
        _chk(c, dt)
        if c.size != n:
            raise ValueError("contributions differ in length")
    out = np.empty(n, out_dtype)
    ptrs = (ctypes.c_void_p * k)(*[c.ctypes.data for c in contrib])
    rc = lib().oracle_reduce_avg(k, ptrs, _dtype_of(contrib[0]), out.ctypes.data,
                                 _dtype_of(out), mode, n)
    if rc:
        raise ValueError("oracle_reduce_avg rejected its arguments")
    return out


def sgd_momentum(a: np.ndarray, w: np.ndarray, v: np.ndarray,
                 lr: float, mu: float, wd: float = 0.0) -> None:
    """In place on w and v."""
    _chk(w, np.float32), _chk(v, np.float32), _chk(a, a.dtype)
    if not (a.size == w.size == v.size):
        raise ValueError("length mismatch")
    rc = lib().oracle_sgd_momentum(a.ctypes.data, _dtype_of(a), w.ctypes.data,
                                   v.ctypes.data, lr, mu, wd, w.size)
    if rc:
        raise ValueError("oracle_sgd_momentum rejected its arguments")


def easgd(x: np.ndarray, c: np.ndarray, alpha: float) -> None:
    """In place on x and c."""
    _chk(x, np.float32), _chk(c, np.float32)
    if x.size != c.size:
        raise ValueError("length mismatch")
    rc = lib().oracle_easgd(x.ctypes.data, c.ctypes.data, alpha, x.size)
    if rc:
        raise ValueError("oracle_easgd rejected its arguments")


def stats(a: np.ndarray):
    """(count of non-finite elements, largest finite magnitude, sum of squares of finite elements)."""
    _chk(a, a.dtype)
    bad, mx, ss = ctypes.c_uint64(0), ctypes.c_float(0), ctypes.c_double(0)
    rc = lib().oracle_stats(a.ctypes.data, _dtype_of(a), a.size, ctypes.byref(bad), ctypes.byref(mx),
                            ctypes.byref(ss))
    if rc:
        raise ValueError("oracle_stats rejected its arguments")
    return int(bad.value), float(mx.value), float(ss.value)


def stats_tensors(ts):
    """The same over a tensor list: counts and squares add up in tensor order, the maximum is the maximum."""
    bad, mx, ss = 0, 0.0, 0.0
    for t in ts:
        b, m, s2 = stats(t)
        bad, mx, ss = bad + b, max(mx, m), ss + s2
    return bad, mx, ss


def stats_ordered_tensors(ts, chunk_elems: int, waves: int, block_chunks: int, combine_threads: int):
    """(non-finite count, largest finite magnitude, sum of squares in the fixed tree order that the four
    parameters define) over a tensor list; see oracle_stats_ordered in the C file for the order."""
    n = len(ts)
    dt = ts[0].dtype
    for t in ts:
        _chk(t, dt)
    ptrs = (ctypes.c_void_p * n)(*[t.ctypes.data if t.size else None for t in ts])
    counts = (ctypes.c_int64 * n)(*[t.size for t in ts])
    bad, mx, ss = ctypes.c_uint64(0), ctypes.c_float(0), ctypes.c_double(0)
    rc = lib().oracle_stats_ordered(n, ptrs, counts, _dtype_of(ts[0]), chunk_elems, waves, block_chunks,
                                    combine_threads, ctypes.byref(bad), ctypes.byref(mx), ctypes.byref(ss))
    if rc:
        raise ValueError("oracle_stats_ordered rejected its arguments")
    return int(bad.value), float(mx.value), float(ss.value)


# -- tensor lists: a plain loop over tensors ---------------------------------------

def pack_fp16_tensors(gs: Sequence[np.ndarray]) -> List[np.ndarray]:
    return [pack_fp16(g) for g in gs]


def unpack_fp16_tensors(hs: Sequence[np.ndarray]) -> List[np.ndarray]:
    return [unpack_fp16(h) for h in hs]


def reduce_avg_tensors(contrib: Sequence[Sequence[np.ndarray]], out_dtype=np.float32,
                       mode: int = AVG) -> List[np.ndarray]:
    """contrib[i][t]: worker i, tensor t."""
    nt = len(contrib[0])
    return [reduce_avg([c[t] for c in contrib], out_dtype, mode) for t in range(nt)]


def sgd_momentum_tensors(a, w, v, lr, mu, wd=0.0) -> None:
    for at, wt, vt in zip(a, w, v):
        sgd_momentum(at, wt, vt, lr, mu, wd)


def easgd_tensors(x, c, alpha) -> None:
    for xt, ct in zip(x, c):
        easgd(xt, ct, alpha)
