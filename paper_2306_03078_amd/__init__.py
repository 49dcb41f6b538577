"""MI355X-native SpQR inference path: thin Python binding over libspqr.so.

Every step of the decode + matvec runs in the HIP kernels of the library; this
package only marshals arguments (PyTorch supplies device memory and streams).
"""
from .binding import (  # noqa: F401
    SpQRError, SpQRMatrix, library_path, load_library, pack_host, packed_bytes,
    spqr_dequant_dense, spqr_gemm_fused, spqr_gemm_fused_ws, spqr_gemm_smallbatch, spqr_gemm_smallbatch_noalloc,
    spqr_gemm_smallbatch_ws, spqr_gemv, spqr_gemv_fused, spqr_gemv_grouped, spqr_pack_check, spqr_plan_batch_steps,
    spqr_set_option, spqr_strerror, spqr_workspace_bytes,
    SPQR_OPT_BATCH_PATH, SPQR_OPT_FORCE_GENERIC, SPQR_OPT_BATCH_STEPS, SPQR_OPT_DENSE_ROWS, SPQR_OPT_GEMV_PLAN,
    SPQR_BATCH_PATH_AUTO, SPQR_BATCH_PATH_VECTOR, SPQR_BATCH_PATH_MATRIX, SPQR_BATCH_PATH_DENSE, SPQR_ERR_WORKSPACE, SPQR_STATIC_SCRATCH_BYTES,
    SPQR_F16, SPQR_F32, SPQR_CHECK_CSR, SPQR_CHECK_NONFINITE, SPQR_CHECK_PERM,
    SPQR_OUT_CODES_U8, SPQR_OUT_DENSE_F16, SPQR_OUT_DENSE_F32, SPQR_OUT_SCALE_F32,
    SPQR_OUT_WITH_OUTLIERS, SPQR_OUT_ZERO_F32, SPQR_LAYOUT_V1, SPQR_LAYOUT_ROUND_ZERO, SPQR_LAYOUT_STATS16,
)
