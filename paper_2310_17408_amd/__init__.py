"""GEMM C = alpha*A*B + beta*C for one MI355X: hand-written HIP/MFMA kernels
behind a C-ABI library, and a thin ctypes binding with the same names."""
from .binding import (  # noqa: F401
    COL_MAJOR,
    ROW_MAJOR,
    F32,
    F16,
    I8,
    GemmError,
    lib_path,
    load,
    gemm_f32,
    gemm_f16,
    gemm_i8,
    gemm_workspace_bytes,
    gemm_status_string,
    gemm_kernel_count,
    gemm_kernel_name,
    gemm_force_kernel,
    gemm_kernel_tile,
    gemm_solo,
    gemm_last_kernel_id,
    gemm_last_split,
)
