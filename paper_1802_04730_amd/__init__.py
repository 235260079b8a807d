"""tc355: MI355X-native evaluation of tensor comprehensions (arXiv 1802.04730).

The package holds the HIP kernels + C-ABI library (csrc/), its thin ctypes
binding (tc355.py), the build driver (build.py) and the seeded synthetic input
generators (inputs.py).  Importing the package touches neither the GPU nor the
shared library; ``paper_1802_04730_amd.tc355`` loads the library on first use
and raises if it is missing.
"""
__all__ = ["inputs", "tc355", "build", "metric"]
