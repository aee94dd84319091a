"""ukst: unified kernel-segregated stride-2 transpose convolution for MI355X (gfx950).

The compute lives in the C-ABI library built from ``csrc/`` (declared in ``include/ukst.h``);
``binding`` is a thin ctypes layer with the same names.  Importing this package never loads the
library; the first call does, and raises if it has not been built.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(__name__ + ".binding")
    raise AttributeError(name)
