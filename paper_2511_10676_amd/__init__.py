"""Pre-attention expert prediction for MoE models on one MI355X (gfx950).

The package is a thin Python binding (`binding`) over a C-ABI HIP library
(`csrc/`, declared in `include/paep.h`), plus the workload table (`configs`)
and the seeded synthetic-input generator (`datagen`).  The library is loaded on
first use; a missing or unbuilt library raises, there is no CPU fallback.
"""
from . import configs, datagen  # noqa: F401

__all__ = ["configs", "datagen", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
