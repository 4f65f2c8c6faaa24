"""SAW-INT4 KV-cache hot path for AMD MI355X: HIP kernels behind a C ABI, plus a thin binding.

``binding`` marshals torch tensors into the C calls of ``include/saw.h``; ``synth`` draws the
seeded synthetic workloads; ``build`` compiles ``csrc/`` into ``libsaw.so`` with hipcc.
"""
from . import build, synth  # noqa: F401  (binding is imported lazily: it needs the built library)

__all__ = ["build", "synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
