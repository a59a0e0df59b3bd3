"""Tile fusion of the matrix chain D = A(BC) on MI355X (gfx950).

Thin Python binding over the C-ABI library `libtilefusion.so` (see include/tilefusion.h).  All
computation happens in the library's HIP kernels; this package only marshals arguments.
PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    TF_F32, TF_F64, TF_FLAG_NO_SPLIT, TF_FLAG_SCHEDULE_ONLY, TF_FLAG_REORDER, TF_FLAG_C_TRANSPOSED,
    TF_FLAG_SKIP_UNREAD, TF_FLAG_NO_BASELINE, TfError, Plan, DeviceCsr, library_path, load_library,
    tf_plan_create, tf_plan_destroy, tf_plan_schedule, tf_plan_workspace, tf_plan_workspace_unfused,
    tf_plan_prepare_unfused, tf_csr_validate, tf_gemm_spmm, tf_gemm_spmm_static, tf_spmm_spmm, tf_unfused_gemm_spmm,
    tf_unfused_spmm_spmm, tf_run_wavefront, tf_last_error, tf_version,
)
