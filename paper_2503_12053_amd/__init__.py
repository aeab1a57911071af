"""MI355X-native iterative gradient compensation + weight update (Ferret, Alg. 1).

Sub-modules:
  workloads  seeded synthetic parameter sets (no arithmetic of the method)
  binding    ctypes binding of the C-ABI library libferret.so (HIP kernels for gfx950)
  build      compiles csrc/ with hipcc

Importing the package loads nothing native; `binding.load()` does and raises if the
library has not been built.
"""
__version__ = "0.1.0"
