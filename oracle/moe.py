"""MoE AllGather + grouped GEMM (paper: kernel list entry for the fused AllGather + group
GEMM, the AllGather+MoE swizzle listing in Appendix "Swizzle", Table "Shapes for
AllGather+MoE").

Tokens are sharded by rank: global token t = s*T_r + i lives on rank s.  Every token
picks top_k experts; assignment f = t*top_k + j goes to expert ids[t, j].  A rank owns the
local experts [e0, e0+E_l), gathers the rows assigned to each of them (grouped by expert,
ascending f inside an expert, which is also ascending source rank) and multiplies each
group by that expert's weight matrix.
"""
import numpy as np

from .formats import decode_bf16
from .schedule import cdiv


def counts_by_rank_by_expert(ids, world, num_experts):
    """count[s, e] = number of assignments of rank s's tokens to expert e.  ids is int32
    [W*T_r, top_k]."""
    tokens, top_k = ids.shape
    t_r = tokens // world
    count = np.zeros((world, num_experts), dtype=np.int64)
    for t in range(tokens):
        for j in range(top_k):
            count[t // t_r, ids[t, j]] += 1
    return count


def route(ids, world, num_experts, expert_begin, num_local_experts):
    """Returns (count [W,E], expert_offset [E_l+1], gather_idx [R]).

    expert_offset is the exclusive prefix sum of the per-expert totals over the local
    experts; gather_idx[expert_offset[j] + q] is the q-th smallest flat assignment index f
    whose expert is expert_begin + j."""
    count = counts_by_rank_by_expert(ids, world, num_experts)
    flat = ids.reshape(-1)
    offsets = [0]
    for j in range(num_local_experts):
        offsets.append(offsets[-1] + int(count[:, expert_begin + j].sum()))
    gather = np.empty(offsets[-1], dtype=np.int64)
    fill = list(offsets[:-1])
    for f in range(flat.shape[0]):
        j = int(flat[f]) - expert_begin
        if 0 <= j < num_local_experts:
            gather[fill[j]] = f
            fill[j] += 1
    return count, np.asarray(offsets, dtype=np.int64), gather


def bisect_right(sorted_vals, x):
    """Number of entries <= x in an ascending list."""
    c = 0
    for v in sorted_vals:
        if v <= x:
            c += 1
    return c


def stage_of_shard(s, rank, world):
    """Delivery position of shard `s` at rank `rank`: the producer of the all-gather delivers the
    rank's own shard first and then walks the ring upwards (rank, rank+1, ... mod world), so shard
    s is the ((s - rank) mod world)-th to arrive."""
    return (s - rank) % world


def tile_schedule(count, expert_begin, num_local_experts, block_m, rank, world):
    """Tile list of the grouped GEMM, ordered by (expert, stage, original tile index).

    Each local expert j with n_j rows has cdiv(n_j, block_m) row tiles.  A tile covering
    rows [q0, q1) of its expert touches the source ranks segment_start..segment_end found
    by bisecting the expert's cumulative per-rank counts.  Its stage is the position, in the
    ring arrival order rank, rank+1, ..., of the last shard it needs.  Inside an expert,
    tiles are emitted by ascending stage; ties keep ascending original index (the paper
    leaves ties to an atomic counter; any order is valid, this one is a function).

    Returns dict of int lists: expert_id, tiled_m (original tile index), segment_start,
    segment_end, stage, and ntiles."""
    n_by_expert = [int(count[:, expert_begin + j].sum()) for j in range(num_local_experts)]
    ntiles_by_expert = [cdiv(n, block_m) for n in n_by_expert]
    acc, run = [], 0
    for v in ntiles_by_expert:
        run += v
        acc.append(run)
    ntiles = run
    rec = []
    for tau in range(ntiles):
        j = bisect_right(acc, tau)
        off_by_expert = acc[j - 1] if j > 0 else 0
        off_in_expert = tau - off_by_expert
        q0 = off_in_expert * block_m
        q1 = min(q0 + block_m, n_by_expert[j])
        cum, run_c = [], 0
        for s in range(world):
            run_c += int(count[s, expert_begin + j])
            cum.append(run_c)
        seg_start = bisect_right(cum, q0)
        seg_end = bisect_right(cum, q1 - 1)
        stage = max(stage_of_shard(s, rank, world) for s in range(seg_start, seg_end + 1))
        rec.append((j, stage, tau, off_by_expert, seg_start, seg_end))
    out = {k: [0] * ntiles for k in ("expert_id", "tiled_m", "segment_start", "segment_end", "stage")}
    for (j, stage, tau, off_by_expert, seg_start, seg_end) in rec:
        before = sum(1 for r in rec if r[0] == j and (r[1] < stage or (r[1] == stage and r[2] < tau)))
        pos = off_by_expert + before
        out["expert_id"][pos] = j
        out["tiled_m"][pos] = tau
        out["segment_start"][pos] = seg_start
        out["segment_end"][pos] = seg_end
        out["stage"][pos] = stage
    out["ntiles"] = ntiles
    return out


def gather_rows(x_shards, gather_idx, top_k):
    """Xg[p, :] = X[gather_idx[p] // top_k, :] with X the row-concatenation of the shards."""
    x = np.concatenate(list(x_shards), axis=0)
    return x[np.asarray(gather_idx) // top_k]


def grouped_gemm(x_shards, ids, w_ekn, world, num_experts, expert_begin, rows=None):
    """Y64 [R, inter]: row p (belonging to local expert j) = Xg[p, :] . W_j in float64.
    w_ekn: bf16 bits of logical weights [E_l, hidden, inter]."""
    num_local = w_ekn.shape[0]
    _, offsets, gather = route(ids, world, num_experts, expert_begin, num_local)
    xg = gather_rows(x_shards, gather, ids.shape[1])
    r_total = int(offsets[-1])
    y = np.zeros((r_total, w_ekn.shape[2]), dtype=np.float64)
    for j in range(num_local):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        if hi > lo:
            y[lo:hi] = decode_bf16(xg[lo:hi]) @ decode_bf16(w_ekn[j])
    return y if rows is None else y[np.asarray(rows)]
