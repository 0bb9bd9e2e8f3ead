"""tdf: tagged static-dataflow execution of recursive function definitions on MI355X.

Thin ctypes binding over libtdf.so (argument marshalling only; every step of an evaluation
runs in the library's HIP kernels).  The library must have been built
(`python -m paper_2410_20225_amd.build`); importing `tdf` fails loudly otherwise.
"""
import importlib

__all__ = ["tdf", "programs", "build"]


def __getattr__(name):
    # submodules load on first use, so that `build` works before the library exists
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
