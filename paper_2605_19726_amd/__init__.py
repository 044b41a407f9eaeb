"""MI355X-native Block Approximate Sparse Attention (BA-Att) hot path.

The compute lives in a C-ABI shared library of hand-written HIP kernels
(`csrc/`, declared in `include/basa.h`); `binding` marshals torch tensors into
it.  Importing the package loads nothing: the library is opened on first use and
a missing or unloadable library raises, there is no fallback path.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(__name__ + ".binding")
    raise AttributeError(name)
