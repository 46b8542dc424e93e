"""Ok-Topk one-GPU hot path for AMD MI355X: thin Python binding over libokt.so.

Importing this package does not load the library; the first call does.  There
is no CPU fallback: without the built HIP library every call raises.
"""
from .binding import (  # noqa: F401
    OktError,
    STREAM_SUM_PARTIALS,
    library_path,
    load_library,
    okt_accumulate_select,
    okt_accumulate_topk_select,
    okt_balance_plan,
    okt_coo_threshold_select,
    okt_debug_slot_min_n,
    okt_debug_spin_limit,
    okt_slot_min_n,
    okt_index_intersect_restore,
    okt_index_intersect_zero,
    okt_last_hip_error,
    okt_region_partition,
    okt_residual_accumulate,
    okt_sparse_reduce,
    okt_sparse_reduce_batch,
    okt_sparse_reduce_batch_workspace_bytes,
    okt_sparse_reduce_segments,
    okt_status_string,
    okt_stream_copy,
    okt_stream_gather,
    okt_stream_sum,
    okt_time_next_kernel,
    okt_threshold_select,
    okt_threshold_select_copy,
    okt_threshold_select_noalloc,
    okt_topk_threshold_exact,
    okt_version,
    okt_workspace_bytes,
)
