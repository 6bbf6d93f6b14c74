"""Seeded synthetic inputs shaped like the paper's workloads.

This package only draws random numbers and packs them into the byte formats the
kernels read (bf16 bit patterns, OCP e4m3 bytes, int32 routing ids).  It holds none
of the method's arithmetic and is the only code shared by the CPU oracle's tests and
the HIP path's tests and benchmark.
"""
from .inputs import (  # noqa: F401
    Config,
    CONFIGS,
    rng_for,
    normal_bf16,
    f32_to_bf16_bits,
    quantize_e4m3,
    integer_bf16,
    routing_topk,
    ag_gemm_inputs,
    gemm_rs_inputs,
    moe_inputs,
    fp8_ag_gemm_inputs,
)
