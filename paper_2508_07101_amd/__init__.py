"""MI355X-native CUSA decode hot path: token selection + sparse attention.

``paper_2508_07101_amd.binding`` is the thin ctypes layer over the C-ABI
library (built from ``csrc/`` by ``paper_2508_07101_amd.build``);
``workloads`` draws seeded synthetic inputs; ``accounting`` holds the
algorithmic byte/flop formulas used for roofline figures.  Submodules are
imported on first use so that drawing inputs never needs the built library.
"""
import importlib

__all__ = ["binding", "workloads", "accounting", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
