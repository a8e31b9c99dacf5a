"""FGMP inference hot path for MI355X: HIP kernels behind a C ABI (csrc/,
include/fgmp.h) and a ctypes binding (fgmp.py).  Importing the package loads
nothing; `fgmp.lib()` loads the shared library on first use."""
