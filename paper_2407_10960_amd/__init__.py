"""lutq: fused lookup-table dequantise + small-batch matmul for MI355X (gfx950).

Thin Python binding over the C ABI of liblutq.so (see include/lutq.h).  The functions here only
marshal arguments: every step of the path runs in the library's HIP kernels (or, for the offline
packer, in its host code).  There is no fallback: if the library is not built, calls raise.
"""
from .binding import (  # noqa: F401
    LutqError,
    Plan,
    lib_path,
    load_library,
    lutq_dequant,
    lutq_matmul,
    lutq_matmul_channel,
    lutq_matmul_pairs,
    lutq_matmul_quads,
    lutq_matmul_static,
    STATIC_SCRATCH_BYTES,
    lutq_pack,
    lutq_packed_bytes,
    lutq_plan_default,
    lutq_plan_default_for,
    lutq_plan_check,
    lutq_pack_layout,
    lutq_plan_table_set,
    lutq_plan_table_lookup,
    lutq_quantize,
    lutq_tune,
    lutq_tune_candidates,
    lutq_unpack,
    lutq_workspace_bytes,
    new_workspace,
    calib_stream_read,
    calib_copy,
    calib_matmul_trace,
    TRACE_STAMPS,
    EXPORTED_SYMBOLS,
)
