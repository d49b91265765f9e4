"""Blockwise parallel decoding on MI355X: thin Python binding over libbpd.so.

The binding only marshals arguments; every step of the method runs in the HIP kernels
behind the C ABI declared in include/bpd.h.  Importing this package does not load the
library; `paper_1811_03115_amd.binding.lib()` does, and fails loudly if it is missing.
"""
__all__ = ["binding", "build"]
