"""MI355X-native library for the draft side of speculative speculative decoding (SSD / Saguaro):
pre-speculation round, speculation-cache lookup and lossless verification as hand-written HIP
kernels behind a C ABI (include/ssd.h).  `binding` is the thin ctypes layer over it; it is loaded on
first use so that `build` can be imported before the library exists.  There is no fallback: using
the package without a built libssd_hip.so raises."""
import importlib

__all__ = ["binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
