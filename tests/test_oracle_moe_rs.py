"""Pins for the MoE down-projection + ReduceScatter oracle: brute force over flat assignments on tiny
inputs, the dense formulation it must equal when the intermediate dimension is split over the ranks, the
special cases that reduce to the grouped GEMM and to the reduce-scatter oracle, and the ordered fp32 combine
against torch's sequential adds."""
import numpy as np
import pytest
import torch

import synth
from oracle import moe, moe_rs, gemm_rs as ors, formats


def _inputs(world, t_r, inter, hidden, experts, top_k, seed=0, integer=False):
    """Tensor-parallel placement: every rank holds all experts and inter / world of the intermediate size.
    Returns ids, h_full [T*top_k, inter] in flat assignment order, w2_full [E, inter, hidden] (bf16 bits)."""
    rng = synth.rng_for(seed, 40, world)
    ids = synth.routing_topk(rng, world * t_r, experts, top_k)
    gen = (lambda shape, std: synth.integer_bf16(rng, shape, -2, 2)) if integer else \
        (lambda shape, std: synth.normal_bf16(rng, shape, std))
    h_full = gen((world * t_r * top_k, inter), 1.0)
    w2_full = gen((experts, inter, hidden), inter ** -0.5)
    return ids, h_full, w2_full


def _rank_slices(ids, h_full, w2_full, world, experts):
    """Per rank: its intermediate slice of the activations, rows in the rank's gathered order, and of W2."""
    i_r = h_full.shape[1] // world
    _, _, gather = moe.route(ids, world, experts, 0, experts)
    hs = [np.ascontiguousarray(h_full[gather][:, r * i_r:(r + 1) * i_r]) for r in range(world)]
    ws = [np.ascontiguousarray(w2_full[:, r * i_r:(r + 1) * i_r, :]) for r in range(world)]
    return hs, ws


@pytest.mark.parametrize("world,t_r,inter,hidden,experts,top_k", [(2, 3, 4, 3, 3, 2), (4, 2, 8, 5, 4, 3), (1, 5, 3, 2, 2, 1)])
def test_equals_the_dense_sum_over_assignments(world, t_r, inter, hidden, experts, top_k):
    """Splitting the intermediate dimension over the ranks and reducing must give, for every token, the plain
    sum over its top_k assignments of gate * (activation row . W2 of its expert): written here with Python
    loops over flat assignments, without the gathered order, the inverse index or the per-rank slices."""
    ids, h_full, w2_full = _inputs(world, t_r, inter, hidden, experts, top_k, seed=3)
    gate = synth.rng_for(5, 40, 1).uniform(0.25, 1.0, size=ids.shape).astype(np.float32)
    hs, ws = _rank_slices(ids, h_full, w2_full, world, experts)
    hd, wd = formats.decode_bf16(h_full), formats.decode_bf16(w2_full)
    want = np.zeros((world * t_r, hidden))
    for t in range(world * t_r):
        for j in range(top_k):
            f = t * top_k + j
            for c in range(hidden):
                want[t, c] += float(gate[t, j]) * sum(hd[f, i] * wd[ids[t, j], i, c] for i in range(inter))
    for d in range(world):
        got = moe_rs.moe_rs(hs, ws, ids, experts, [0] * world, d, gate)
        assert np.allclose(got, want[d * t_r:(d + 1) * t_r], rtol=1e-12, atol=1e-12)
    # a dropped gate, a transposed weight or a wrong inverse index all change the result
    assert not np.allclose(moe_rs.moe_rs(hs, ws, ids, experts, [0] * world, 0, None), want[:t_r])


def test_special_cases_reduce_to_known_oracles():
    world, t_r, inter, hidden, experts = 4, 6, 8, 5, 3
    # top_k = 1, no gate, one rank: the combine is a permutation of the grouped down-projection
    ids, h_full, w2_full = _inputs(1, world * t_r, inter, hidden, experts, 1, seed=7)
    _, offsets, gather = moe.route(ids, 1, experts, 0, experts)
    h = h_full[gather]
    y = moe_rs.down_proj(h, w2_full, offsets)
    z = moe_rs.partial(h, w2_full, ids, 1, experts, 0)
    assert np.array_equal(z[gather], y)                       # row p of y is token gather[p]
    assert np.array_equal(moe_rs.inverse_index(gather, gather.size)[gather], np.arange(gather.size))
    # experts sharded over ranks instead (2 local experts each): an assignment is served by exactly one rank,
    # so the reduce-scatter of the partials is the reduce-scatter oracle's sum of the same blocks
    world, experts, top_k = 3, 6, 2
    ids, h_full, w2_full = _inputs(world, t_r, inter, hidden, experts, top_k, seed=9)
    hs, ws, e0 = [], [], []
    for r in range(world):
        _, _, g = moe.route(ids, world, experts, 2 * r, 2)
        hs.append(np.ascontiguousarray(h_full[g]))
        ws.append(np.ascontiguousarray(w2_full[2 * r:2 * r + 2]))
        e0.append(2 * r)
    parts = [moe_rs.partial(hs[r], ws[r], ids, world, experts, e0[r]) for r in range(world)]
    full = moe_rs.partial(h_full[moe.route(ids, world, experts, 0, experts)[2]], w2_full, ids, world, experts, 0)
    assert np.allclose(sum(parts), full, rtol=1e-12, atol=1e-12)
    for d in range(world):
        assert np.allclose(moe_rs.moe_rs(hs, ws, ids, experts, e0, d), full[d * t_r:(d + 1) * t_r], rtol=1e-12, atol=1e-12)
    # an assignment whose expert is not on the rank adds nothing there
    pos = moe_rs.inverse_index(moe.route(ids, world, experts, 2, 2)[2], ids.size)
    assert ((pos >= 0) == ((ids.reshape(-1) >= 2) & (ids.reshape(-1) < 4))).all()


def test_ordered_combine_matches_torch_sequential_adds():
    tokens, top_k, hidden, experts = 40, 3, 16, 5
    rng = synth.rng_for(11, 40, 2)
    ids = synth.routing_topk(rng, tokens, experts, top_k)
    _, offsets, gather = moe.route(ids, 1, experts, 1, 3)           # experts 1..3 local: some assignments missing
    y_bits = synth.normal_bf16(rng, (int(offsets[-1]), hidden), 2.0)
    gate = (2.0 ** rng.integers(-2, 2, size=ids.shape)).astype(np.float32)
    for g in (None, gate):
        got = moe_rs.combine_f32_ordered(y_bits, gather, tokens, top_k, g)
        y = torch.from_numpy(y_bits.view(np.int16)).view(torch.bfloat16).float()
        pos = moe_rs.inverse_index(gather, tokens * top_k)
        acc = torch.zeros((tokens, hidden), dtype=torch.float32)
        for j in range(top_k):
            for t in range(tokens):
                p = pos[t * top_k + j]
                if p >= 0:
                    acc[t] = acc[t] + (1.0 if g is None else float(g[t, j])) * y[p]
        want = acc.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, want)
        exact = moe_rs.combine(formats.decode_bf16(y_bits), gather, tokens, top_k, g)
        ulp = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7
        assert np.all(np.abs(formats.decode_bf16(got) - exact) <= ulp)
