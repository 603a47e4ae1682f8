"""MI355X-native forward path of one SLiM-compressed linear layer.

The work is done by hand-written HIP kernels behind a C-ABI shared library
(csrc/, declared in include/slim.h); `binding` marshals torch tensors into it.
Importing the package does not load the library; the first call does, and it
raises if the library has not been built.
"""
from . import accounting, workloads  # noqa: F401

__all__ = ["accounting", "workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
