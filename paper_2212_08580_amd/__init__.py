"""Nested gradient coding on one MI355X: C-ABI library `libngc` + a thin binding.

`libngc` (the ctypes binding in paper_2212_08580_amd/ngc.py) exposes the calls of the coded
gradient path: partition gradients, layered encode, decode-vector selection and
decode.  `workloads` draws the seeded synthetic inputs.  Nothing here computes
on the CPU in place of the GPU kernels: if the HIP library is not built the
binding raises.
"""
__all__ = ["workloads"]
