"""MI355X-native ring-step attention (the per-device hot path of Double-Ring-Attention).

`binding` mirrors the C ABI of libloong.so one to one; `ring` replays one rank's
micro-steps on a single GPU.  The HIP library is loaded on first use of anything but the
build module, and that fails if it has not been built (python -m paper_2406_18485_amd.build):
there is no fallback implementation.
"""
import importlib

_LAZY_SUBMODULES = ("binding", "ring", "build")


def __getattr__(name):
    # `build` must be importable before the library exists; everything else comes from the
    # binding, which loads libloong.so (ImportError if it is missing).
    if name in _LAZY_SUBMODULES:
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
