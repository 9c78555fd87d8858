"""MI355X-native SD-KDE hot path: hand-written HIP kernels behind a C ABI (libsdkde.so) and a
thin ctypes binding with the same entry-point names."""
from .binding import (
    SDKDE_ETOOLARGE, SDKDE_FLAG_MAX_SHIFT, SDKDE_FLAG_SAMPLES_PREPARED, SDKDE_FLAG_SYMMETRIC, SDKDE_PREC_FP16X2, SDKDE_PREC_FP16X2_ALL, SDKDE_PREC_FP32, SDKDE_STATIC_SCRATCH_BYTES, SdkdeError, load,
    make_workspace, sdkde_debias, sdkde_describe_plan, sdkde_eval, sdkde_eval_laplace, sdkde_fit_eval, sdkde_fit_eval_static,
    sdkde_profile_enable, sdkde_profile_summary, sdkde_score, sdkde_status_string, sdkde_workspace_bytes,
    workspace_bytes_any_precision,
)

__all__ = [
    "SDKDE_ETOOLARGE", "SDKDE_FLAG_MAX_SHIFT", "SDKDE_FLAG_SAMPLES_PREPARED", "SDKDE_STATIC_SCRATCH_BYTES", "SDKDE_FLAG_SYMMETRIC", "SDKDE_PREC_FP16X2", "SDKDE_PREC_FP16X2_ALL", "SDKDE_PREC_FP32", "SdkdeError", "load",
    "make_workspace", "sdkde_debias", "sdkde_describe_plan", "sdkde_eval", "sdkde_eval_laplace", "sdkde_fit_eval", "sdkde_fit_eval_static",
    "sdkde_profile_enable", "sdkde_profile_summary", "sdkde_score", "sdkde_status_string", "sdkde_workspace_bytes",
    "workspace_bytes_any_precision",
]
