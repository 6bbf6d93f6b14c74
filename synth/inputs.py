"""Seeded input generators for the five benchmark configurations and their scaled-down
test variants.

Every array returned here is raw storage: uint16 bf16 bit patterns, uint8 OCP e4m3
bytes, int32 routing ids, float32 scales.  Consumers decode the bytes themselves (the
oracle in software, the kernels in hardware), so nothing here is on the parity path.

Streams: numpy PCG64 seeded with SeedSequence([seed, cfg_id, tensor_id]) so that each
tensor of each configuration has its own reproducible stream.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Config:
    """One workload.  Field meaning depends on `kind`:

    ag_gemm / ag_gemm_fp8 : world, rank, m_per_rank, n, k
    gemm_rs               : world, rank, m (= world * rows per rank), n, k  (k is the local K)
    moe                   : world, rank, tokens_per_rank, hidden (k), inter (n),
                            num_experts, top_k, num_local_experts
    """
    cfg_id: int
    kind: str
    world: int
    rank: int
    m_per_rank: int = 0
    n: int = 0
    k: int = 0
    tokens_per_rank: int = 0
    num_experts: int = 0
    top_k: int = 0
    num_local_experts: int = 0
    seed: int = 0

    @property
    def m(self) -> int:
        return self.world * self.m_per_rank

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS: Dict[int, Config] = {
    # smoke: W=2, 2 x [128,256] @ [256,256]
    1: Config(1, "ag_gemm", world=2, rank=0, m_per_rank=128, n=256, k=256),
    # Llama-70B-like MLP up-projection at TP=8: [8192,8192] @ [8192,3584]
    2: Config(2, "ag_gemm", world=8, rank=0, m_per_rank=1024, n=3584, k=8192),
    # matching down-projection: [8192,3584] @ [3584,8192], reduce-scattered over 8 ranks
    3: Config(3, "gemm_rs", world=8, rank=0, m_per_rank=1024, n=8192, k=3584),
    # MoE: 8 x 1024 tokens, hidden 4096, 64 experts top-2, 8 local experts, inter 1536
    4: Config(4, "moe", world=8, rank=0, tokens_per_rank=1024, k=4096, n=1536,
              num_experts=64, top_k=2, num_local_experts=8),
    # decode: 8 x [16,8192] fp8 @ [8192,8192] fp8
    5: Config(5, "ag_gemm_fp8", world=8, rank=0, m_per_rank=16, n=8192, k=8192),
}


def rng_for(seed: int, cfg_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg_id, tensor_id])))


# --------------------------------------------------------------------------- packing
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); returns uint16 bits.
    Inputs are finite, so no NaN handling is needed."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def normal_bf16(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return f32_to_bf16_bits(x)


def integer_bf16(rng: np.random.Generator, shape, lo: int = -2, hi: int = 2) -> np.ndarray:
    """Small integers stored as bf16: products and (short) sums of these are exact in
    fp32 and in bf16, which lets a test demand bit-equal outputs."""
    v = rng.integers(lo, hi + 1, size=shape).astype(np.float32)
    return f32_to_bf16_bits(v)


def quantize_e4m3(x: np.ndarray, scale: np.ndarray | float) -> np.ndarray:
    """Encode x/scale as OCP e4m3 bytes (4 exponent bits, bias 7, 3 mantissa bits, finite
    only, largest magnitude 448), round to nearest even, saturating.  Used only to make
    input bytes; the consumers decode those bytes on their own."""
    y = (np.asarray(x, dtype=np.float64) / np.asarray(scale, dtype=np.float64))
    sign = np.signbit(y)
    a = np.minimum(np.abs(y), 448.0)
    # exponent of the binade, clamped to the subnormal binade 2^-6
    m, e = np.frexp(a)                    # a = m * 2^e, m in [0.5, 1)
    e = e - 1                             # a = (2m) * 2^e, 2m in [1, 2)
    e = np.maximum(e, -6)
    step = np.ldexp(1.0, e - 3)           # spacing of representable values in that binade
    q = np.rint(a / step)                 # numpy rint is round-half-even
    val = q * step                        # may have carried to the next binade: still exact
    val = np.minimum(val, 448.0)
    # now encode val exactly
    m2, e2 = np.frexp(val)
    e2 = e2 - 1
    normal = val >= 2.0 ** -6
    exp_field = np.where(normal, e2 + 7, 0).astype(np.int64)
    mant = np.where(normal, np.rint((val / np.ldexp(1.0, e2) - 1.0) * 8.0),
                    np.rint(val / 2.0 ** -9)).astype(np.int64)
    code = (exp_field << 3) | mant
    code = np.where(val == 0.0, 0, code)
    code = code | (sign.astype(np.int64) << 7)
    return code.astype(np.uint8)


def routing_topk(rng: np.random.Generator, tokens: int, num_experts: int, top_k: int) -> np.ndarray:
    """For every token, top_k distinct experts drawn uniformly without replacement, kept
    in draw order.  int32 [tokens, top_k]."""
    keys = rng.random(size=(tokens, num_experts))
    order = np.argsort(keys, axis=1, kind="stable")
    return np.ascontiguousarray(order[:, :top_k]).astype(np.int32)


# --------------------------------------------------------------------------- workloads
def ag_gemm_inputs(cfg: Config, integer: bool = False):
    """AllGather-GEMM inputs: W shards A_s [m_per_rank,k] ~ N(0,1) and logical B [k,n]
    ~ N(0, 1/k), both bf16.  Returns (a_shards list of uint16, b_kn uint16)."""
    a = []
    for s in range(cfg.world):
        r = rng_for(cfg.seed, cfg.cfg_id, 100 + s)
        a.append(integer_bf16(r, (cfg.m_per_rank, cfg.k)) if integer
                 else normal_bf16(r, (cfg.m_per_rank, cfg.k)))
    r = rng_for(cfg.seed, cfg.cfg_id, 1)
    b = integer_bf16(r, (cfg.k, cfg.n)) if integer else normal_bf16(r, (cfg.k, cfg.n), cfg.k ** -0.5)
    return a, b


def gemm_rs_inputs(cfg: Config, integer: bool = False):
    """GEMM-ReduceScatter inputs for every emulated rank s: A_s [m,k] ~ N(0,1), logical
    B_s [k,n] ~ N(0,1/k), bf16.  Returns (a_list, b_list)."""
    a, b = [], []
    for s in range(cfg.world):
        ra = rng_for(cfg.seed, cfg.cfg_id, 100 + s)
        rb = rng_for(cfg.seed, cfg.cfg_id, 200 + s)
        if integer:
            a.append(integer_bf16(ra, (cfg.m, cfg.k)))
            b.append(integer_bf16(rb, (cfg.k, cfg.n), -1, 1))
        else:
            a.append(normal_bf16(ra, (cfg.m, cfg.k)))
            b.append(normal_bf16(rb, (cfg.k, cfg.n), cfg.k ** -0.5))
    return a, b


def moe_inputs(cfg: Config, integer: bool = False):
    """MoE inputs: W token shards X_s [tokens_per_rank, hidden] ~ N(0,1) bf16, routing ids
    int32 [W*tokens_per_rank, top_k], local expert weights as logical [E_l, hidden, inter]
    ~ N(0, 1/hidden) bf16.  Local experts are [rank*E_l, rank*E_l + E_l)."""
    xs = []
    for s in range(cfg.world):
        r = rng_for(cfg.seed, cfg.cfg_id, 100 + s)
        xs.append(integer_bf16(r, (cfg.tokens_per_rank, cfg.k)) if integer
                  else normal_bf16(r, (cfg.tokens_per_rank, cfg.k)))
    ids = routing_topk(rng_for(cfg.seed, cfg.cfg_id, 2), cfg.world * cfg.tokens_per_rank,
                       cfg.num_experts, cfg.top_k)
    r = rng_for(cfg.seed, cfg.cfg_id, 1)
    shape = (cfg.num_local_experts, cfg.k, cfg.n)
    w = integer_bf16(r, shape, -1, 1) if integer else normal_bf16(r, shape, cfg.k ** -0.5)
    return xs, ids, w


def fp8_ag_gemm_inputs(cfg: Config):
    """Decode-shaped fp8 AllGather-GEMM: A shards are N(0,1) quantised with one scale per
    shard (amax/448), logical B [k,n] is N(0,1/k) quantised with one scale per column.
    Returns (a_shards uint8, a_scales f32[W], b_kn uint8, b_scales f32[n])."""
    a, sa = [], np.empty(cfg.world, dtype=np.float32)
    for s in range(cfg.world):
        x = rng_for(cfg.seed, cfg.cfg_id, 100 + s).standard_normal(
            size=(cfg.m_per_rank, cfg.k), dtype=np.float32)
        sa[s] = np.float32(np.abs(x).max() / 448.0)
        a.append(quantize_e4m3(x, float(sa[s])))
    wf = rng_for(cfg.seed, cfg.cfg_id, 1).standard_normal(size=(cfg.k, cfg.n), dtype=np.float32)
    wf *= np.float32(cfg.k ** -0.5)
    sb = (np.abs(wf).max(axis=0) / 448.0).astype(np.float32)
    b = quantize_e4m3(wf, sb[None, :].astype(np.float64))
    return a, sa, b, sb
