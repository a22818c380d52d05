"""MI355X-native decode hot path behind ODMA contiguous KV allocation.

``paper_2512_09427_amd.binding`` is the ctypes layer over ``libodma.so``; it is
imported on first use so that ``paper_2512_09427_amd.build`` can run before the
library exists.  There is no CPU fallback: using the package without the built
library raises ImportError.
"""
import importlib

__all__ = ["binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
