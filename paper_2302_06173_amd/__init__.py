"""MI355X-native update-undo library (Swift, arXiv 2302.06173, section "Update-undo").

  binding   ctypes wrappers with the names of the C entry points (include/swift_undo.h)
  build     compiles csrc/api.hip into libswift_undo.so for gfx950
  synth     seeded synthetic workloads (shapes and value distributions only)

The binding is imported lazily so that `python -m paper_2302_06173_amd.build` works before the
library exists; using it without a built library raises ImportError (there is no fallback).
"""
import importlib

__all__ = ["binding", "build", "synth"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
