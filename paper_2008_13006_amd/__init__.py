"""Tile-wise (TW) sparse GEMM for MI355X (gfx950).

``workloads`` draws the seeded synthetic inputs; ``binding`` is the thin ctypes layer over the
C-ABI library ``libtw.so`` (HIP kernels + host packer).  ``binding`` is imported on first use so
that the input generators stay importable on a machine where the library has not been built;
using any GEMM entry point without the built library raises.
"""
from . import workloads  # noqa: F401


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
