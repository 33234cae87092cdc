"""Judge Q KV-cache eviction hot path (arXiv 2509.10798, Section 4.3) for AMD MI355X.

The work is done by hand-written HIP kernels in ``libjq.so`` (sources under
``csrc/``, C ABI in ``include/jq.h``); this package is the thin Python binding.
"""
from .binding import (  # noqa: F401
    EXPORTS, STATIC_WS_BYTES, TRACE_KERNELS, TRACE_MARKS, JQError, Pages, Shape, alloc_workspace, compact, compact_inplace, copy_probe, evict, evict_inplace, evict_paged, evict_paged_inplace, evict_static, evict_stream, hit_rate, lib, map_mse, map_mse_fused, pool, reload_knobs, score, score_paged, select_topk,
    status_string, workspace_bytes,
)
