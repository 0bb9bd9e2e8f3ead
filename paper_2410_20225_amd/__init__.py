"""tdf: tagged static-dataflow execution of recursive function definitions on MI355X.

Thin ctypes binding over libtdf.so (argument marshalling only; every step of an evaluation
runs in the library's HIP kernels).  The library must have been built
(`python -m paper_2410_20225_amd.build`); importing `tdf` fails loudly otherwise.
"""
from . import tdf  # noqa: F401
from . import programs  # noqa: F401
