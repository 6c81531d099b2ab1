"""libshiftadd: the ShiftAddViT block hot path as hand-written HIP kernels for gfx950.

The package holds the C-ABI library (csrc/, built in-tree as libshiftadd.so),
a thin ctypes binding with the same names (binding.py) and the seeded input
generators (workloads.py).  Importing the package loads nothing; the first
call into the binding loads the library and fails loudly if it is missing.
"""
from __future__ import annotations


def load_library():
    from . import binding
    return binding.load_library()


def __getattr__(name):
    if name.startswith("sa_") or name in ("binding", "SAError"):
        import importlib
        binding = importlib.import_module(__name__ + ".binding")
        if name == "binding":
            return binding
        return getattr(binding, name)
    raise AttributeError(name)
