"""ctypes binding of libpxchg.so.  Same names as the C ABI (include/pxchg.h);
each function only converts its arguments and checks the returned status."""
from __future__ import annotations

import ctypes
import os
import sys
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpxchg.so")

AVG, SUM = 0, 1
F32, F16 = 0, 1
MAX_K = 64
OPT_CHUNK_ELEMS, OPT_BLOCKS_PER_CU, OPT_CHECK_RANGES, OPT_NONTEMPORAL, OPT_CENTER_RESIDENT = 0, 1, 2, 3, 4
OPT_ALL_POLICIES_BUILT = 5
TABLE_OPTION_INHERIT = -2
ERR_IN_USE = 7

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_int = ctypes.c_int
_f = ctypes.c_float
_pp = ctypes.POINTER(_vp)

# name -> (restype, argtypes); also the list of symbols the header declares
SIGNATURES = {
    "pxchg_status_string": (ctypes.c_char_p, [_int]),
    "pxchg_version": (_int, []),
    "pxchg_set_option": (_int, [_int, _i64]),
    "pxchg_get_option": (_i64, [_int]),
    "pxchg_plan_chunks": (_int, [_int, ctypes.POINTER(_i64), _i64, _i64, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(_i64)]),
    "pxchg_plan_groups": (_int, [_int, ctypes.POINTER(_i64), _i64, _int, _int, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(_int)]),
    "pxchg_table_create": (_int, [_int, ctypes.POINTER(_i64), _pp]),
    "pxchg_table_destroy": (_int, [_vp]),
    "pxchg_table_view": (_int, [_vp, _int, _int, _pp]),
    "pxchg_table_set_multipliers": (_int, [_vp, ctypes.POINTER(_f), ctypes.POINTER(_f)]),
    "pxchg_table_set_option": (_int, [_vp, _int, _i64]),
    "pxchg_table_get_option": (_i64, [_vp, _int]),
    "pxchg_table_total": (_i64, [_vp]),
    "pxchg_table_n_tensors": (_int, [_vp]),
    "pxchg_table_n_chunks": (_i64, [_vp]),
    "pxchg_bufset_create": (_int, [_vp, _int, _pp, _pp]),
    "pxchg_bufset_destroy": (_int, [_vp]),
    "pxchg_pack_fp16": (_int, [_vp, _int, _pp, _pp, _vp]),
    "pxchg_unpack_fp16": (_int, [_vp, _int, _pp, _pp, _vp]),
    "pxchg_reduce_avg": (_int, [_vp, _int, _pp, _vp, _int, _vp]),
    "pxchg_sgd_momentum": (_int, [_vp, _vp, _vp, _vp, _f, _f, _f, _vp]),
    "pxchg_easgd": (_int, [_vp, _vp, _vp, _f, _vp]),
    "pxchg_easgd_round": (_int, [_vp, _int, _pp, _vp, _f, _vp]),
    "pxchg_reduce_avg_sgd_momentum": (_int, [_vp, _int, _pp, _int, _int, _vp, _vp, _f, _f, _f, _vp]),
    "pxchg_buffer_stats": (_int, [_vp, _vp, _vp, _vp]),
    "pxchg_buffer_stats_static": (_int, [_vp, _vp, _vp, _vp]),
}


class Stats(ctypes.Structure):
    """Host mirror of pxchg_stats (24 bytes)."""
    _fields_ = [("nonfinite", ctypes.c_uint64), ("sum_sq", ctypes.c_double), ("max_abs", ctypes.c_float),
                ("reserved", ctypes.c_uint32)]


class PxchgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib: Optional[ctypes.CDLL] = None


def library_path() -> str:
    return _LIB_PATH


def open_library(path: str) -> ctypes.CDLL:
    """Load a build of the library from `path` and declare its signatures.  Besides the regular libpxchg.so
    this serves the tuning build (every cache policy compiled in), which tests and measurements load next to
    it: tables and buffer sets remember the library that made them."""
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_1605_08325_amd.build` "
            "(hipcc, gfx950); this package has no CPU or eager fallback")
    try:
        # torch first: it brings a HIP runtime of its own, and the library must bind to the same one, or the two
        # runtimes do not know each other's allocations (every call then answers "no usable GPU")
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


def load() -> ctypes.CDLL:
    """The library that new tables are made with: libpxchg.so, loaded on first use.  Raises if it has not been
    built: there is no fallback."""
    global _lib
    if _lib is None:
        _lib = open_library(_LIB_PATH)
    return _lib


class using:
    """Context manager: inside it, new tables (and set_option / get_option) go to `lib`, a library returned by
    open_library()."""

    def __init__(self, lib: ctypes.CDLL):
        self._new = lib

    def __enter__(self):
        global _lib
        self._old, _lib = _lib, self._new
        return self._new

    def __exit__(self, *exc):
        global _lib
        _lib = self._old
        return False


def status_string(status: int) -> str:
    return load().pxchg_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise PxchgError(status, where)


def version() -> int:
    return int(load().pxchg_version())


def set_option(option: int, value: int) -> None:
    _check(load().pxchg_set_option(option, value), "pxchg_set_option")


def get_option(option: int) -> int:
    return int(load().pxchg_get_option(option))


def plan_chunks(counts: Sequence[int], chunk_elems: int) -> Tuple[List[int], List[int], List[int]]:
    """Host-only: (tensor, start, len) of every chunk."""
    lib = load()
    n = len(counts)
    c = (_i64 * max(n, 1))(*counts)
    total = _i64(0)
    _check(lib.pxchg_plan_chunks(n, c, chunk_elems, 0, None, None, None, ctypes.byref(total)), "pxchg_plan_chunks")
    m = total.value
    t = (ctypes.c_int32 * max(m, 1))()
    s = (_i64 * max(m, 1))()
    ln = (ctypes.c_int32 * max(m, 1))()
    _check(lib.pxchg_plan_chunks(n, c, chunk_elems, m, t, s, ln, ctypes.byref(total)), "pxchg_plan_chunks")
    return list(t[:m]), list(s[:m]), list(ln[:m])


def plan_groups(counts: Sequence[int], min_elems: int, reverse: bool = True, lib=None) -> List[Tuple[int, int]]:
    """Host-only: (first tensor, number of tensors) of every group of pxchg_plan_groups."""
    lib = lib or load()
    n = len(counts)
    c = (_i64 * max(n, 1))(*counts)
    total = _int(0)
    _check(lib.pxchg_plan_groups(n, c, int(min_elems), int(bool(reverse)), 0, None, None, ctypes.byref(total)),
           "pxchg_plan_groups")
    m = total.value
    first, num = (ctypes.c_int32 * max(m, 1))(), (ctypes.c_int32 * max(m, 1))()
    _check(lib.pxchg_plan_groups(n, c, int(min_elems), int(bool(reverse)), m, first, num, ctypes.byref(total)),
           "pxchg_plan_groups")
    return [(int(first[i]), int(num[i])) for i in range(m)]


def _stream_ptr(stream) -> Optional[int]:
    """None -> torch's current stream; an int is taken as a hipStream_t."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# Destruction waits for the device and frees device memory, which would invalidate a stream capture in progress.
# Python decides by itself when an object dies (a collector run can fall into the middle of a capture), so a
# handle that dies while this thread's current stream is capturing is put aside and destroyed later.
_deferred: List = []


def _capturing() -> bool:
    torch = sys.modules.get("torch")
    try:
        return bool(torch is not None and torch.cuda.is_available() and torch.cuda.is_current_stream_capturing())
    except Exception:
        return False


def flush_deferred() -> int:
    """Destroys what was put aside (during captures, or a table whose views or sets were still alive when the
    collector took it first); returns how many handles that were.  Called by itself whenever an object is
    destroyed outside a capture."""
    n = 0
    if _capturing():
        return n
    pending, _deferred[:] = list(_deferred), []
    # buffer sets and views before the tables they belong to
    for lib, fname, handle in sorted(pending, key=lambda item: item[1] == "pxchg_table_destroy"):
        if getattr(lib, fname)(handle) == ERR_IN_USE:
            _deferred.append((lib, fname, handle))
        else:
            n += 1
    return n


def _destroy(lib, fname: str, handle) -> None:
    if _capturing():
        _deferred.append((lib, fname, handle))
        return
    flush_deferred()
    if getattr(lib, fname)(handle) == ERR_IN_USE:
        _deferred.append((lib, fname, handle))      # retried when the next object dies


class Table:
    """pxchg_table: element counts of the parameter set's tensors."""

    def __init__(self, counts: Sequence[int]):
        self.counts = [int(c) for c in counts]
        self._h = _vp()
        self._lib = load()
        arr = (_i64 * max(len(self.counts), 1))(*self.counts)
        _check(self._lib.pxchg_table_create(len(self.counts), arr, ctypes.byref(self._h)), "pxchg_table_create")

    @property
    def handle(self):
        return self._h

    @property
    def total(self) -> int:
        return int(self._lib.pxchg_table_total(self._h))

    @property
    def n_tensors(self) -> int:
        return int(self._lib.pxchg_table_n_tensors(self._h))

    @property
    def n_chunks(self) -> int:
        return int(self._lib.pxchg_table_n_chunks(self._h))

    def set_multipliers(self, lr_mult: Optional[Sequence[float]] = None,
                        wd_mult: Optional[Sequence[float]] = None) -> None:
        """Per-tensor learning-rate and decay multipliers for the update calls (None = all ones)."""
        def arr(x):
            if x is None:
                return None
            if len(x) != len(self.counts):
                raise ValueError("one multiplier per tensor expected")
            return (_f * len(x))(*[float(v) for v in x])
        _check(self._lib.pxchg_table_set_multipliers(self._h, arr(lr_mult), arr(wd_mult)), "pxchg_table_set_multipliers")

    def set_option(self, option: int, value: int) -> None:
        """pxchg_table_set_option: this table's own cache policy or center-resident switch
        (TABLE_OPTION_INHERIT: back to the process-wide setting)."""
        _check(self._lib.pxchg_table_set_option(self._h, option, value), "pxchg_table_set_option")

    def get_option(self, option: int) -> int:
        return int(self._lib.pxchg_table_get_option(self._h, option))

    def bufset(self, tensors, dtype: Optional[int] = None) -> "BufSet":
        return BufSet(self, tensors, dtype)

    def view(self, first_tensor: int, n_tensors: int) -> "Table":
        """pxchg_table_view: a handle for tensors first_tensor .. first_tensor + n_tensors - 1, to be used with
        this table's buffer sets.  The view keeps this table alive."""
        v = Table.__new__(Table)
        v.counts = self.counts[first_tensor:first_tensor + n_tensors]
        v._h = _vp()
        v._lib = self._lib
        v._parent = self
        _check(self._lib.pxchg_table_view(self._h, int(first_tensor), int(n_tensors), ctypes.byref(v._h)),
               "pxchg_table_view")
        return v

    def bucketed_views(self, min_elems: int, reverse: bool = True) -> List["Table"]:
        """One view per group of pxchg_plan_groups: runs of consecutive tensors with at least `min_elems` elements
        (the last group formed holds what is left), by default formed from the last tensor backwards, the order
        in which back-propagation produces gradients."""
        return [self.view(f, m) for f, m in plan_groups(self.counts, min_elems, reverse, self._lib)]

    def close(self) -> None:
        if self._h:
            _destroy(self._lib, "pxchg_table_destroy", self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class BufSet:
    """pxchg_bufset: one device pointer per tensor.  `tensors` is a sequence of
    torch CUDA tensors (kept alive by this object) or of raw device addresses
    (then `dtype` is required)."""

    def __init__(self, table: Table, tensors, dtype: Optional[int] = None):
        self.table = table
        self._keep = None
        ptrs = []
        if len(tensors) != len(table.counts):
            raise ValueError("one tensor per table entry expected")
        if all(isinstance(t, int) for t in tensors):
            if dtype is None:
                raise ValueError("dtype is required with raw addresses")
            ptrs = [int(t) for t in tensors]
        else:
            import torch
            want = None
            for t, c in zip(tensors, table.counts):
                if not t.is_cuda or not t.is_contiguous() or t.numel() != c:
                    raise ValueError("contiguous CUDA tensors with the table's element counts expected")
                d = {torch.float32: F32, torch.float16: F16}.get(t.dtype)
                if d is None or (want is not None and d != want):
                    raise ValueError("all tensors must be float32, or all float16")
                want = d
                ptrs.append(t.data_ptr() if c else 0)
            if dtype is not None and dtype != want:
                raise ValueError("dtype does not match the tensors")
            dtype = want
            self._keep = list(tensors)
        self.dtype = dtype
        self._h = _vp()
        arr = (_vp * max(len(ptrs), 1))(*[p or None for p in ptrs])
        self._lib = table._lib
        _check(self._lib.pxchg_bufset_create(table.handle, dtype, arr, ctypes.byref(self._h)), "pxchg_bufset_create")

    @property
    def handle(self):
        return self._h

    @property
    def tensors(self):
        return self._keep

    def close(self) -> None:
        if self._h:
            _destroy(self._lib, "pxchg_bufset_destroy", self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _handles(sets: Sequence[BufSet]):
    return (_vp * max(len(sets), 1))(*[s.handle for s in sets])


def pack_fp16(table: Table, src_f32: Sequence[BufSet], dst_f16: Sequence[BufSet], stream=None) -> None:
    if len(src_f32) != len(dst_f16):
        raise ValueError("as many destinations as sources expected")
    _check(table._lib.pxchg_pack_fp16(table.handle, len(src_f32), _handles(src_f32), _handles(dst_f16),
                                  _stream_ptr(stream)), "pxchg_pack_fp16")


def unpack_fp16(table: Table, src_f16: Sequence[BufSet], dst_f32: Sequence[BufSet], stream=None) -> None:
    if len(src_f16) != len(dst_f32):
        raise ValueError("as many destinations as sources expected")
    _check(table._lib.pxchg_unpack_fp16(table.handle, len(src_f16), _handles(src_f16), _handles(dst_f32),
                                    _stream_ptr(stream)), "pxchg_unpack_fp16")


def reduce_avg(table: Table, contrib: Sequence[BufSet], out: BufSet, mode: int = AVG, stream=None) -> None:
    _check(table._lib.pxchg_reduce_avg(table.handle, len(contrib), _handles(contrib), out.handle, mode,
                                   _stream_ptr(stream)), "pxchg_reduce_avg")


def sgd_momentum(table: Table, grad: BufSet, param: BufSet, vel: BufSet, lr: float, mu: float,
                 wd: float = 0.0, stream=None) -> None:
    _check(table._lib.pxchg_sgd_momentum(table.handle, grad.handle, param.handle, vel.handle, lr, mu, wd,
                                     _stream_ptr(stream)), "pxchg_sgd_momentum")


def easgd(table: Table, x: BufSet, c: BufSet, alpha: float, stream=None) -> None:
    _check(table._lib.pxchg_easgd(table.handle, x.handle, c.handle, alpha, _stream_ptr(stream)), "pxchg_easgd")


def easgd_round(table: Table, x: Sequence[BufSet], c: BufSet, alpha: float, stream=None) -> None:
    _check(table._lib.pxchg_easgd_round(table.handle, len(x), _handles(x), c.handle, alpha, _stream_ptr(stream)),
           "pxchg_easgd_round")


def reduce_avg_sgd_momentum(table: Table, contrib: Sequence[BufSet], param: BufSet, vel: BufSet, lr: float,
                            mu: float, wd: float = 0.0, mode: int = AVG, wire_dtype: int = F32,
                            stream=None) -> None:
    _check(table._lib.pxchg_reduce_avg_sgd_momentum(table.handle, len(contrib), _handles(contrib), mode, wire_dtype,
                                                param.handle, vel.handle, lr, mu, wd, _stream_ptr(stream)),
           "pxchg_reduce_avg_sgd_momentum")


def buffer_stats(table: Table, bufset: BufSet, out, stream=None) -> None:
    """`out`: a CUDA tensor of at least 24 bytes (e.g. 3 int64), or a raw device address.  Read it back with
    read_stats() after synchronising."""
    addr = out if isinstance(out, int) else out.data_ptr()
    if not isinstance(out, int) and out.numel() * out.element_size() < ctypes.sizeof(Stats):
        raise ValueError("the output needs 24 bytes")
    _check(table._lib.pxchg_buffer_stats(table.handle, bufset.handle, addr, _stream_ptr(stream)), "pxchg_buffer_stats")


def buffer_stats_static(table: Table, bufset: BufSet, out, stream=None) -> None:
    """pxchg_buffer_stats_static: the same result, with the partial results in the library's static device array
    (nothing allocated, by this call or for it)."""
    addr = out if isinstance(out, int) else out.data_ptr()
    if not isinstance(out, int) and out.numel() * out.element_size() < ctypes.sizeof(Stats):
        raise ValueError("the output needs 24 bytes")
    _check(table._lib.pxchg_buffer_stats_static(table.handle, bufset.handle, addr, _stream_ptr(stream)),
           "pxchg_buffer_stats_static")


def read_stats(out) -> Tuple[int, float, float]:
    """(nonfinite, max_abs, sum_sq) from the tensor buffer_stats() wrote; copies 24 bytes to the host."""
    raw = out.view(-1).cpu().numpy().tobytes()[:ctypes.sizeof(Stats)]
    st = Stats.from_buffer_copy(raw)
    return int(st.nonfinite), float(st.max_abs), float(st.sum_sq)
