"""kvswap_hip: the KVSwap decode-step hot path as HIP kernels for MI355X (gfx950).

The package is a thin binding over the C-ABI library built from csrc/: argument
marshalling only, every step of the path runs in the library's kernels.  There
is no CPU fallback; a missing or unloadable library raises.
"""
from .binding import (  # noqa: F401
    KVS_F32, KVS_BF16, KVS_FP8_E4M3, KVS_REDUCE_MAX, KVS_REDUCE_MEAN, KVS_HEADS_SEPARATE, KVS_HEADS_JOINT,
    KvsError, Params, load_library, library_path,
    kvs_check_params, kvs_workspace_bytes, kvs_workspace_init, kvs_workspace_check, kvs_set_wait_limit, kvs_status_str, kvs_version, kvs_last_device_error,
    kvs_build_metadata, kvs_build_metadata_rows, kvs_append_group,
    kvs_predict_select, kvs_predict_scores, kvs_select_topk,
    kvs_sparse_decode_attn, kvs_sparse_decode_attn_rb, kvs_sparse_decode_attn_paged,
    kvs_selection_overlap, kvs_decode_step, kvs_decode_step_rb, kvs_decode_step_static, kvs_decode_step_single_launch, kvs_attend_select_next, kvs_attend_select_next_rb,
    KVS_STATIC_SCRATCH_BYTES,
)
