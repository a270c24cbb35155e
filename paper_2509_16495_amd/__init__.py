"""One GPU's share of an attention layer under Shift Parallelism (arXiv 2509.16495) for MI355X.

`binding` wraps the C ABI of libshiftattn.so (hand-written gfx950 kernels); `workloads` draws the
seeded synthetic inputs; `build` compiles the library.  Importing the package is cheap; the
binding (and torch) load on first use.
"""
import importlib

__all__ = ["binding", "workloads", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
