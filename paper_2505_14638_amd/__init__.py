"""MI355X-native W4A8 quantized linear layer (INT4 weights, FP8 E4M3 compute) of arXiv 2505.14638.

The package holds the HIP kernels behind a C-ABI library (csrc/, built by `build.py`), a thin
ctypes binding with the same entry-point names (`binding.py`) and the seeded synthetic workload
generators (`synthetic.py`).  Importing the package loads nothing; `binding.lib()` loads the
library and raises if it has not been built.
"""
__all__ = ["binding", "build", "synthetic"]
