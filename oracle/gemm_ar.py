"""GEMM + AllReduce (paper, Appendix "GEMM All-Reduce": host launcher, the persistent GEMM
that notifies per tile, and the all-reduce consumer).

Rank s holds A_s [M, K_l] and B_s [K_l, N] (its slice of the contraction dimension) and
computes the partial P_s = A_s . B_s into a buffer every rank can read; a tile of P_s is
announced by one flag per (rank, tile).  Every rank ends with the same full matrix
C = sum_s P_s  [M, N].  Overlap changes when a tile is reduced, never its value.
"""
import numpy as np

from .formats import decode_bf16, encode_bf16_rne
from .schedule import cdiv, grouped_order, xcd_remap


def partial_bits(a, b_kn):
    """The buffer a rank publishes: P = A . B rounded once to bf16 (storage bits); the
    launcher allocates that buffer in the input dtype."""
    return encode_bf16_rne((decode_bf16(a) @ decode_bf16(b_kn)).astype(np.float32))


def gemm_ar(a_list, b_list, rows=None):
    """C64 [M, N] (or the given rows of it) in float64 from every rank's bf16 inputs: the
    plain definition, the sum over ranks of the partial products."""
    m = a_list[0].shape[0]
    idx = np.arange(m) if rows is None else np.asarray(rows)
    out = np.zeros((len(idx), b_list[0].shape[1]), dtype=np.float64)
    for a, b in zip(a_list, b_list):
        out += decode_bf16(a[idx]) @ decode_bf16(b)
    return out


def allreduce_partials_f32_ordered(partials):
    """The reduction as the consumer is specified to do it here: the published bf16 tiles of
    ranks 0..W-1 added in that order in fp32, one round-to-nearest-even.  bf16 bits."""
    acc = decode_bf16(partials[0]).astype(np.float32)
    for p in partials[1:]:
        acc = (acc + decode_bf16(p).astype(np.float32)).astype(np.float32)
    return encode_bf16_rne(acc)


def tile_flag_index(pid_m, pid_n, num_pid_n):
    """Index of a tile's flag inside one rank's flag array (persistent GEMM listing, last
    lines): row-major over the tile grid."""
    return pid_m * num_pid_n + pid_n


def tile_at_position(position, m, n, block_m, block_n, group_m, num_xcd=0, per_xcd=0):
    """Tile at `position` of the GEMM's tile order: the grouped order of the persistent GEMM
    listing (its `_compute_pid`).  num_xcd > 0 adds the chiplet remap of this build (blocks of
    num_xcd * per_xcd positions, a run of consecutive tile ids per chiplet).  -> (pid_m, pid_n)"""
    npm, npn = cdiv(m, block_m), cdiv(n, block_n)
    ntiles = npm * npn
    assert 0 <= position < ntiles
    tile_id = xcd_remap(position, ntiles, num_xcd, per_xcd) if num_xcd else position
    return grouped_order(tile_id, npm, npn, group_m)


def persistent_tile(position, m, n, block_m, block_n, group_m, gemm_wgs, num_xcd=0):
    """The paper's persistent form of the same order: `gemm_wgs` work-groups loop over the tiles,
    work-group g taking positions g, g+G, g+2G, ... (the range with step NUM_GEMM_SMS).  With the
    chiplet remap a round of G positions is one remap block.
    Returns (pid_m, pid_n, work-group, round)."""
    ntiles = cdiv(m, block_m) * cdiv(n, block_n)
    assert not num_xcd or gemm_wgs % num_xcd == 0 or ntiles <= gemm_wgs   # a round is a whole number of chiplet runs
    pid_m, pid_n = tile_at_position(position, m, n, block_m, block_n, group_m, num_xcd,
                                    cdiv(gemm_wgs, num_xcd) if num_xcd else 0)
    return pid_m, pid_n, position % gemm_wgs, position // gemm_wgs


def two_shot_owner(position, world):
    """Two-shot form (the consumer listing's broadcast branch): the rank that reduces the tile at
    `position` of the tile order and broadcasts it.  The listing deals blocks of NUM_COMM_SMS consecutive
    tiles to the ranks in turn; with blocks of one tile that is position mod world."""
    return position % world
