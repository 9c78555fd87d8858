"""MI355X-native SD-KDE hot path: hand-written HIP kernels behind a C ABI (libsdkde.so) and a
thin ctypes binding with the same entry-point names."""
from .binding import (SdkdeError, load, make_workspace, sdkde_debias, sdkde_eval, sdkde_eval_laplace, sdkde_profile_enable,
                      sdkde_profile_summary, sdkde_score, sdkde_status_string, sdkde_workspace_bytes)

__all__ = ["SdkdeError", "load", "make_workspace", "sdkde_debias", "sdkde_eval", "sdkde_eval_laplace", "sdkde_profile_enable",
           "sdkde_profile_summary", "sdkde_score", "sdkde_status_string", "sdkde_workspace_bytes"]
