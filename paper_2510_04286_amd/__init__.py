"""SliceMoE layer forward pass for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI.

    paper_2510_04286_amd.binding   ctypes binding with the entry points of include/slicemoe.h
    paper_2510_04286_amd.workload  seeded synthetic inputs (no method arithmetic)
    paper_2510_04286_amd.build     compiles csrc/*.hip into libslicemoe.so

Importing the package loads nothing heavy; `binding` pulls in torch and the shared library.
"""
import importlib

__all__ = ["binding", "workload", "build"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
