"""MI355X-native hot path of HEART's sparse-attention step (gfx950 HIP kernels
behind a C ABI).  `binding` mirrors the four entry points of include/heart.h on
torch-ROCm tensors; it only marshals arguments -- every step runs in the HIP
kernels, and importing/calling it without the built library fails loudly."""
from .binding import (  # noqa: F401
    HEART_ATTN_FOLD_SCALE,
    HeartError,
    HeartShape,
    heart_attn_workspace_bytes,
    heart_block_sparse_attn,
    heart_block_sparse_attn_flags,
    heart_block_sparse_attn_static,
    heart_drift,
    heart_ebc_band_error,
    heart_ebc_select,
    heart_ebc_workspace_bytes,
    heart_last_error,
    heart_mask_topp,
    heart_mask_topp_workspace_bytes,
    heart_mask_topp_ws,
    heart_pool_drift,
    heart_pool_drift_workspace_bytes,
    heart_pool_qk,
    heart_scores_antidiag,
    heart_scores_antidiag_workspace_bytes,
    heart_ubench_copy,
    heart_ubench_read,
    heart_ubench_mfma_bf16,
    heart_version,
    heart_workspace_bytes,
    lib_path,
    load_library,
)
