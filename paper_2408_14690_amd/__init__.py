"""MI355X-native TEAL decode path: thresholded sparse GEMV behind a C ABI.

The work is done by libteal.so (hand-written HIP for gfx950, include/teal.h).
This package only marshals arguments; PyTorch supplies device memory and
streams.  There is no CPU fallback: without the built library every call
raises.
"""
from .binding import (  # noqa: F401
    TEAL_OK, TEAL_ERR_NULL, TEAL_ERR_SHAPE, TEAL_ERR_ALIGN, TEAL_ERR_THRESHOLD,
    TEAL_ERR_WORKSPACE, TEAL_ERR_UNSUPPORTED, TEAL_ERR_HIP, TEAL_ERR_STATIC_LIMIT,
    TealError, check, library_path, load_library, prepare,
    teal_status_string, teal_version, teal_workspace_bytes,
    teal_sparsify, teal_sparse_gemv_bf16, teal_sparse_gemv_bf16_ex,
    teal_sparse_gemv_w8, teal_sparse_gemv_w4, teal_pack_bf16, teal_pack_bf16_pitch, teal_gemv_plan,
    teal_sparse_gemv_bf16_multi, teal_abs_histogram, teal_histogram_thresholds, TEAL_HIST_BINS,
    teal_workspace_bytes_batch, teal_sparsify_batch, teal_sparse_gemv_bf16_batch,
    teal_sparse_gemv_bf16_batch_ex, TEAL_MAX_BATCH, teal_sparse_gemv_w8_multi,
    teal_sparse_gemv_w4_multi, teal_swiglu_f16, teal_sparse_gemv_bf16_swiglu,
    teal_sparse_gemv_bf16_batch_multi, teal_gemv_plan_multi, teal_survivors_offset,
    teal_rmsnorm_f16, teal_sparse_gemv_bf16_rmsnorm_multi, teal_workspace_bytes_stack,
    teal_sparse_gemv_bf16_stack, teal_sparse_gemv_w8_stack, teal_sparse_gemv_w4_stack,
    teal_stream_read_probe, teal_sparse_gemv_w8_swiglu, teal_sparse_gemv_w8_rmsnorm_multi,
    teal_sparse_gemv_w4_swiglu, teal_sparse_gemv_w4_rmsnorm_multi,
    teal_static_scratch_limit, teal_static_scratch_init, teal_sparse_gemv_bf16_static,
    MlpShape, teal_workspace_bytes_mlp, teal_mlp_down_region_offset, teal_mlp_status_offset,
    teal_mlp_plan, teal_mlp_block_info, teal_sparse_mlp_bf16, teal_sparse_mlp_w8, teal_sparse_mlp_w4,
    teal_sparse_gemv_bf16_multi_pitch, teal_sparse_gemv_w8_multi_pitch, teal_gemv_plan_multi_pitch,
    teal_sparse_gemv_bf16_rmsnorm_multi_pitch,
)
