"""GEMM-ReduceScatter (paper, Appendix "GEMM Reduce-Scatter": host launcher, producer
kernel and the reduce-scatter listing).

Rank s holds A_s [M, K_l] and B_s [K_l, N] (its slice of the contraction dimension) and
computes the partial P_s = A_s . B_s.  Rank d's output is its row block of the sum:
out_d = sum_s P_s[d*M_r:(d+1)*M_r, :], M_r = M / W.
"""
import numpy as np

from .formats import decode_bf16, encode_bf16_rne


def partial(a, b_kn):
    """P = A . B in float64 from bf16 storage bits."""
    return decode_bf16(a) @ decode_bf16(b_kn)


def gemm_rs(a_list, b_list, rank):
    """out_rank [M_r, N] in float64 from every rank's bf16 inputs."""
    world = len(a_list)
    m = a_list[0].shape[0]
    assert m % world == 0
    m_r = m // world
    n = b_list[0].shape[1]
    out = np.zeros((m_r, n), dtype=np.float64)
    for s in range(world):
        out += decode_bf16(a_list[s][rank * m_r:(rank + 1) * m_r]) @ decode_bf16(b_list[s])
    return out


def arrival_order(rank, world):
    """Order in which peers' partial blocks reach `rank`.  Rank s starts its tile rows at
    segment s+1 and walks upward, so it finishes segment d at step (d-s-1) mod W: the
    block of rank d-1 arrives first, then d-2, ..., and the rank's own block is last."""
    return [(rank - 1 - i) % world for i in range(world)]


def reduce_slots_f64(slots):
    """Exact sum of the W bf16 partial blocks (storage bits) in float64."""
    acc = np.zeros(slots[0].shape, dtype=np.float64)
    for s in slots:
        acc += decode_bf16(s)
    return acc


def reduce_slots_f32_ordered(slots):
    """The reduction as the kernel is specified to do it: fp32 accumulation in slot order
    0..W-1 starting from slot 0, one round-to-nearest-even to bf16.  Returns bf16 bits."""
    acc = decode_bf16(slots[0]).astype(np.float32)
    for s in slots[1:]:
        acc = (acc + decode_bf16(s).astype(np.float32)).astype(np.float32)
    return encode_bf16_rne(acc)


def fused_scatter_row(m_row, rank, world, m):
    """Where row `m_row` of rank `rank`'s partial product goes when the scatter is fused into the GEMM's
    stores (producer kernel, FUSE_SCATTER branch): (destination rank, row in that rank's [M, N] buffer).
    The destination is the owner of the row's segment; inside its buffer the row lands in the slot of the
    sending rank, at the row's offset inside the segment."""
    m_r = m // world
    return m_row // m_r, rank * m_r + m_row % m_r
