"""libpxchg for MI355X: the per-GPU arithmetic of a data-parallel parameter
exchange (pack to half precision, fixed-order sum and average, momentum-SGD
update, elastic averaging), as hand-written gfx950 kernels behind a C ABI.

This package is only the thin Python face of ``libpxchg.so``: argument
marshalling, nothing else.  There is no CPU fallback: if the shared library has
not been built (``python -m paper_1605_08325_amd.build``) every call raises.
"""
from .binding import (  # noqa: F401
    AVG, SUM, F32, F16, MAX_K,
    OPT_CHUNK_ELEMS, OPT_BLOCKS_PER_CU, OPT_CHECK_RANGES, OPT_NONTEMPORAL, OPT_CENTER_RESIDENT,
    OPT_ALL_POLICIES_BUILT, TABLE_OPTION_INHERIT, ERR_IN_USE, open_library, using,
    PxchgError, Table, BufSet,
    load, library_path, version, set_option, get_option, plan_chunks, plan_groups, status_string,
    pack_fp16, unpack_fp16, reduce_avg, sgd_momentum, easgd, easgd_round,
    reduce_avg_sgd_momentum, buffer_stats, buffer_stats_static, read_stats, Stats, flush_deferred,
)
