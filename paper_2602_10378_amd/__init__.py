"""MI355X-native SD-KDE hot path: hand-written HIP kernels behind a C ABI (libsdkde.so) and a
thin ctypes binding with the same entry-point names."""
from . import binding as _binding

# every entry point and constant of include/sdkde.h under its own name, plus the binding's helpers
__all__ = sorted(name for name in vars(_binding) if name.startswith(("sdkde_", "SDKDE_"))) + [
    "SdkdeError", "load", "make_workspace", "workspace_bytes_any_precision"]
globals().update({name: getattr(_binding, name) for name in __all__})
