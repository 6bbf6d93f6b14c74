"""MI355X-native fused communication + GEMM kernels (AllGather-GEMM, GEMM-ReduceScatter,
MoE AllGather + grouped GEMM) behind a C ABI, with a thin ctypes binding.

Importing this package does not load the shared library; `paper_2605_02953_amd.binding`
does, and raises if it has not been built (`python -m paper_2605_02953_amd.build`).
"""
__all__ = ["binding", "build"]
