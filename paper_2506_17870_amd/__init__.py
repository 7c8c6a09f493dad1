"""NestQuant nested-integer hot path for AMD MI355X (gfx950): hand-written HIP kernels
behind a C ABI (include/nq.h) with a thin ctypes binding.  PyTorch is used only for device
memory and streams.

The binding (and with it libnq.so) is loaded on first use of any attribute, so that
`python -m paper_2506_17870_amd.build` can run before the library exists; using the package
without a built library raises ImportError -- there is no fallback path.
"""
import importlib

__all__ = ["binding", "build", "inputs"]


def __getattr__(name):
    if name in ("build", "inputs", "binding"):
        return importlib.import_module(f"{__name__}.{name}")
    binding = importlib.import_module(f"{__name__}.binding")
    try:
        return getattr(binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
