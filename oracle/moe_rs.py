"""MoE down-projection + ReduceScatter (paper: workload "MoE+ReduceScatter" of the evaluation, Table
"MoE+RS performance"; tensor-parallel placement of Table "Summary of Parallelism": every rank holds every
expert's weights for its slice of the intermediate dimension).

The paper gives the workload and its shape, not a listing; the definition used here is the plain one.
Tokens are sharded by rank (token t = s*T_r + i on rank s); assignment f = t*top_k + j goes to expert
ids[t, j].  Rank r holds, for every assignment routed to one of its experts, the activation row h_r[p, :]
(its slice of the intermediate dimension), rows grouped by expert in the order of moe.route (position p
of assignment gather_idx[p]), and the experts' down-projection weights W2_r [E_l, I_r, H].  Then

    y_r[p, :]  = h_r[p, :] . W2_r[expert(p)]                       (grouped GEMM)
    z_r[t, :]  = sum_j  g[t, j] * y_r[pos(t*top_k + j), :]          (top-k combine; g = 1 when no gate
                                                                     weights are given; assignments whose
                                                                     expert is not on the rank add nothing)
    out_d[i,:] = sum_r z_r[d*T_r + i, :]                            (reduce-scatter over the ranks)
"""
import numpy as np

from .formats import decode_bf16, encode_bf16_rne
from . import moe


def inverse_index(gather_idx, num_assignments):
    """pos[f] = position of assignment f among the gathered rows, -1 if its expert is not local."""
    pos = np.full(num_assignments, -1, dtype=np.int64)
    for p, f in enumerate(np.asarray(gather_idx)):
        pos[int(f)] = p
    return pos


def down_proj(h, w2_eih, expert_offsets):
    """y64 [R, H]: row p (expert j) = h[p, :] . W2[j] in float64.  h: bf16 bits [R, I]; w2: bf16 bits of the
    logical weights [E_l, I, H]."""
    r_total = int(expert_offsets[-1])
    y = np.zeros((r_total, w2_eih.shape[2]), dtype=np.float64)
    for j in range(w2_eih.shape[0]):
        lo, hi = int(expert_offsets[j]), int(expert_offsets[j + 1])
        if hi > lo:
            y[lo:hi] = decode_bf16(h[lo:hi]) @ decode_bf16(w2_eih[j])
    return y


def combine(y, gather_idx, tokens, top_k, gate=None):
    """z [tokens, H] = sum over a token's assignments (in order j = 0..top_k-1) of gate * y[pos]; float64."""
    pos = inverse_index(gather_idx, tokens * top_k)
    z = np.zeros((tokens, y.shape[1]), dtype=np.float64)
    for t in range(tokens):
        for j in range(top_k):
            p = pos[t * top_k + j]
            if p >= 0:
                z[t] += (1.0 if gate is None else float(gate[t, j])) * y[p]
    return z


def partial(h, w2_eih, ids, world, num_experts, expert_begin, gate=None):
    """One rank's z [tokens, H] in float64 from its bf16 inputs."""
    _, offsets, gather = moe.route(ids, world, num_experts, expert_begin, w2_eih.shape[0])
    return combine(down_proj(h, w2_eih, offsets), gather, ids.shape[0], ids.shape[1], gate)


def moe_rs(h_list, w2_list, ids, num_experts, expert_begin_list, rank, gate=None):
    """out_rank [T_r, H] in float64: the rank's row block of the sum over ranks of their partials."""
    world = len(h_list)
    t_r = ids.shape[0] // world
    out = None
    for s in range(world):
        z = partial(h_list[s], w2_list[s], ids, world, num_experts, expert_begin_list[s], gate)
        blk = z[rank * t_r:(rank + 1) * t_r]
        out = blk if out is None else out + blk
    return out


def combine_f32_ordered(y_bits, gather_idx, tokens, top_k, gate=None):
    """The combine as the kernel is specified to do it: the bf16 rows of y, fp32 accumulation
    acc = fma(gate, y, acc) over j = 0..top_k-1 starting from 0, one round-to-nearest-even to bf16.
    Exact here for gate = None or gates that are powers of two (every product is then exact in fp32).
    Returns bf16 bits [tokens, H]."""
    pos = inverse_index(gather_idx, tokens * top_k)
    y = decode_bf16(y_bits).astype(np.float32)
    acc = np.zeros((tokens, y.shape[1]), dtype=np.float32)
    for j in range(top_k):
        p = pos[np.arange(tokens) * top_k + j]
        rows = np.where(p >= 0)[0]
        g = np.float32(1.0) if gate is None else gate[rows, j].astype(np.float32)[:, None]
        acc[rows] = (acc[rows] + (g * y[p[rows]]).astype(np.float32)).astype(np.float32)
    return encode_bf16_rne(acc)
