"""MI355X-native ECO optimizer step (HIP library libeco.so + thin ctypes binding).

The binding is loaded on first use, so that ``paper_2601_22101_amd.build`` can be imported before the
library exists.  There is no CPU or PyTorch fallback: if libeco.so is missing, using the package raises.
"""
import importlib

__all__ = ["binding", "build", "harness"]


def __getattr__(name):
    if name in ("binding", "harness", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    b = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(b, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
