"""Certified quantized decode attention for MI355X: HIP library + ctypes binding.

`paper_2605_20868_amd.binding` holds the calls (same names as include/cqa.h).
The binding is imported on first use so that the build step can run before the
shared library exists; any use without the built library raises ImportError.
"""
import importlib

__all__ = ["binding", "build"]


def __getattr__(name):
    if name in ("binding", "build"):
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
