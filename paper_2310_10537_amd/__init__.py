"""MX cast and MX GEMM for MI355X (gfx950): hand-written HIP kernels behind a
C-ABI library, with a thin ctypes binding (see binding.py).

Importing the package loads nothing; the shared library is opened on the first
call into the binding and a missing library is an error, never a fallback.
"""
