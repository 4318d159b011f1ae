"""UniSparse hot path for MI355X (gfx950): composite-token proxy, block selection and
block-sparse attention as hand-written HIP kernels behind a C-ABI library.

``workloads`` (numpy-only input generators) imports without the native library;
``api`` is the thin binding over ``libunisparse.so`` and raises if it is not built.
"""
__version__ = "0.1.0"
