"""MI355X-native training path of the uniformly-sparse extreme-classification output layer.

`usl` is the binding of the C-ABI library (HIP kernels for gfx950); `build` compiles it.
Importing the package does not load the library; `from paper_2306_03725_amd import usl` does,
and raises if it has not been built.
"""
__all__ = ["usl", "build"]
