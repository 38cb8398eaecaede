"""Fused GEMM + activation + row-normalisation for MI355X (gfx950): hand-written HIP kernels
behind a C ABI (include/fge.h), with a thin ctypes binding (binding.py) and the seeded
synthetic-input generator (inputs.py).  Importing the package loads nothing; the library is
loaded on the first call."""
