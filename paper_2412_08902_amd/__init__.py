"""hcspmm: hybrid MFMA / vector-ALU SpMM for graph adjacency matrices on AMD MI355X.

Thin Python binding over the C-ABI library ``libhcspmm.so`` (see ``include/hcspmm.h``).
The binding only marshals arguments; every step of the method runs in the HIP kernels.
There is no CPU fallback: if the library is missing the import of :mod:`.binding` fails.
"""
from ._build import build_library, LIB_PATH  # noqa: F401

__all__ = ["build_library", "LIB_PATH", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
