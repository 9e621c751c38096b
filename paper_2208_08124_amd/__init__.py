"""Packed variable-length fused multi-head attention for MI355X (gfx950).

The compute lives in a C-ABI HIP library (csrc/); `fmha` holds the ctypes
binding.  Nothing is loaded at import time so that the input generator in
`workloads` can be used on machines without a GPU.
"""
