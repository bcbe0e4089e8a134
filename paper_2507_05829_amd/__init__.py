"""Banded local-operator chains (Intra-DP local operation parallelism) on MI355X.

The product is liblop.so (HIP kernels + C ABI, see include/lop.h); ``lop`` is its ctypes
binding. Importing ``paper_2507_05829_amd.lop`` raises if the library has not been built.
"""
