"""AllGather-GEMM (paper, Appendix "AllGather GEMM": the host launcher's docstring and the
producer / consumer listings).

Definition: every rank holds a row shard A_s [M_r, K]; the gathered matrix places shard s
at rows [s*M_r, (s+1)*M_r); the local output is C = gathered(A) . B with B logically
[K, N].  Overlap changes when a tile is computed, never its value, so the oracle is the
plain product in fp64.
"""
import numpy as np

from .formats import decode


def gather(a_shards):
    """Row placement of the all-gather: shard s -> rows [s*M_r, (s+1)*M_r)."""
    world = len(a_shards)
    m_r, k = a_shards[0].shape
    out = np.empty((world * m_r, k), dtype=a_shards[0].dtype)
    for s in range(world):
        assert a_shards[s].shape == (m_r, k)
        out[s * m_r:(s + 1) * m_r, :] = a_shards[s]
    return out


def arrival_order(rank, world):
    """Order in which the producer delivers shards to `rank`: its own first, then the
    ring (rank+1, rank+2, ...), as in the full-mesh pull producer."""
    return [(rank + i) % world for i in range(world)]


def ag_gemm(a_shards, b_kn, dtype="bf16", a_scales=None, b_scales=None, rows=None):
    """C64 [M, N] = gather(A) . B in float64.

    a_shards: list of W arrays of storage bits [M_r, K]; b_kn: storage bits of logical B
    [K, N]; dtype "bf16" or "e4m3".  For e4m3 the product is scaled by
    a_scales[row // M_r] * b_scales[col].  `rows` restricts the result to those rows of C.
    """
    a = gather(a_shards)
    m_r = a_shards[0].shape[0]
    idx = np.arange(a.shape[0]) if rows is None else np.asarray(rows)
    a64 = decode(a[idx], dtype)
    b64 = decode(b_kn, dtype)
    c = a64 @ b64
    if a_scales is not None:
        c = c * np.asarray(a_scales, dtype=np.float64)[idx // m_r][:, None]
    if b_scales is not None:
        c = c * np.asarray(b_scales, dtype=np.float64)[None, :]
    return c
