"""MI355X (gfx950) dense GEMM, C = alpha*op(A)*op(B) + beta*C, behind a C ABI.

The arithmetic lives in the HIP library ``libpeak_gemm.so`` (see
``include/peak_gemm.h`` and ``include/peak_calib.h``); this package only marshals arguments.  There is no
CPU fallback: if the library is not built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    PEAK_DT_F32, PEAK_DT_F16, PEAK_DT_BF16,
    PEAK_OK, PEAK_ERR_INVALID_ARG, PEAK_ERR_UNSUPPORTED, PEAK_ERR_WORKSPACE, PEAK_ERR_HIP, PEAK_ERR_ALLOC,
    PEAK_BIAS_NONE, PEAK_BIAS_PER_COLUMN, PEAK_BIAS_PER_ROW, PEAK_ACT_NONE, PEAK_ACT_RELU, PEAK_ACT_GELU_TANH, PEAK_GEMM_C_F32,
    PEAK_GEMM_STREAMK_ON, PEAK_GEMM_STREAMK_OFF,
    PeakGemmDesc, PeakGemmEpilogue, PeakError, lib_path, load_library,
    peak_gemm_create, peak_gemm_workspace_bytes, peak_gemm_run, peak_gemm_run_fused, peak_gemm_run_static,
    PEAK_GEMM_STATIC_WORKSPACE_BYTES, peak_gemm_destroy,
    peak_status_string, peak_gemm_plan_info, peak_gemm_variant_count, peak_gemm_variant_name,
    peak_gemm_load_tuning, peak_calib_mfma, peak_calib_read, peak_calib_lds_load, force_flags, Plan,
)
