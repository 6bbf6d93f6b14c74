"""Pins for the GEMM + AllReduce oracle: brute force on tiny inputs, the identity with a
single GEMM over the concatenated contraction dimension, all-reduce = all-gather of the
reduce-scatter, a printed closed form, and the invariants of the persistent tile schedule."""
import numpy as np
import pytest
import torch

import synth
from oracle import gemm_ar as oar, gemm_rs as ors, ag_gemm as oag, formats, schedule as osch


def _brute_matmul(a, b):
    m, k = a.shape
    n = b.shape[1]
    c = np.zeros((m, n))
    for i in range(m):
        for j in range(n):
            s = 0.0
            for t in range(k):
                s += float(a[i, t]) * float(b[t, j])
            c[i, j] = s
    return c


def _bf(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


@pytest.mark.parametrize("world,m,k,n", [(2, 4, 3, 2), (4, 8, 2, 3), (3, 3, 5, 4)])
def test_brute_force_over_concatenated_contraction(world, m, k, n):
    rng = np.random.default_rng(world * 10 + k)
    a_list = [synth.normal_bf16(rng, (m, k)) for _ in range(world)]
    b_list = [synth.normal_bf16(rng, (k, n)) for _ in range(world)]
    a_cat = np.concatenate([formats.decode_bf16(a) for a in a_list], axis=1)
    b_cat = np.concatenate([formats.decode_bf16(b) for b in b_list], axis=0)
    got = oar.gemm_ar(a_list, b_list)
    assert got.shape == (m, n)
    assert np.allclose(got, _brute_matmul(a_cat, b_cat), rtol=1e-13, atol=1e-13)
    assert np.array_equal(oar.gemm_ar(a_list, b_list, rows=[m - 1, 0]), got[[m - 1, 0]])


def test_closed_form_detects_dropped_rank_and_transposition():
    # rank s: A_s[m, 0] = m + 1, B_s[0, n] = (s + 1)(n + 1)  ->  C[m, n] = (m+1)(n+1) * W(W+1)/2
    world, m, k, n = 4, 3, 2, 5
    a_list, b_list = [], []
    for s in range(world):
        a = np.zeros((m, k), dtype=np.float32)
        a[:, 0] = np.arange(1, m + 1)
        b = np.zeros((k, n), dtype=np.float32)
        b[0, :] = (s + 1) * np.arange(1, n + 1)
        a_list.append(_bf(a))
        b_list.append(_bf(b))
    want = np.outer(np.arange(1, m + 1), np.arange(1, n + 1)) * (world * (world + 1) // 2)
    assert np.array_equal(oar.gemm_ar(a_list, b_list), want)


def test_allreduce_is_allgather_of_reducescatter_and_world1_is_gemm():
    cfg = synth.CONFIGS[3].scaled(world=4, m_per_rank=3, k=16, n=8)
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    full = oar.gemm_ar(a_list, b_list)
    for d in range(cfg.world):
        assert np.allclose(full[d * 3:(d + 1) * 3], ors.gemm_rs(a_list, b_list, d), rtol=1e-14, atol=1e-14)
    one = oar.gemm_ar(a_list[:1], b_list[:1])
    assert np.array_equal(one, oag.ag_gemm([a_list[0]], b_list[0]))


def test_published_partial_is_one_bf16_rounding_of_the_product():
    cfg = synth.CONFIGS[3].scaled(world=2, m_per_rank=8, k=64, n=16)
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    bits = oar.partial_bits(a_list[0], b_list[0])
    a_t = torch.from_numpy(a_list[0].view(np.int16).copy()).view(torch.bfloat16).double()
    b_t = torch.from_numpy(b_list[0].view(np.int16).copy()).view(torch.bfloat16).double()
    ref = (a_t @ b_t).float().to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    # integers: nothing is rounded, and the ordered fp32 all-reduce of the partials is the exact sum
    ia, ib = synth.gemm_rs_inputs(cfg, integer=True)
    parts = [oar.partial_bits(a, b) for a, b in zip(ia, ib)]
    assert np.array_equal(formats.decode_bf16(oar.allreduce_partials_f32_ordered(parts)), oar.gemm_ar(ia, ib))


def test_ordered_allreduce_matches_sequential_fp32_adds():
    rng = np.random.default_rng(11)
    parts = [synth.normal_bf16(rng, (5, 24)) for _ in range(8)]
    t = [torch.from_numpy(p.view(np.int16).copy()).view(torch.bfloat16).float() for p in parts]
    acc = t[0].clone()
    for x in t[1:]:
        acc = acc + x
    ref = acc.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oar.allreduce_partials_f32_ordered(parts), ref)
    # a different order may round differently, the exact sum bounds both
    exact = sum(formats.decode_bf16(p) for p in parts)
    got = formats.decode_bf16(oar.allreduce_partials_f32_ordered(parts))
    assert np.max(np.abs(got - exact) / np.maximum(np.abs(exact), 1e-3)) < 2 ** -7


@pytest.mark.parametrize("m,n,bm,bn,group_m,wgs,xcd", [
    (1024, 1024, 256, 256, 4, 8, 0),        # two rounds of eight
    (8192, 8192, 256, 256, 8, 224, 8),      # five rounds, the last one partial
    (1000, 520, 128, 128, 8, 16, 8),        # ragged edges
    (300, 200, 128, 128, 8, 256, 8),        # fewer tiles than work-groups
])
def test_persistent_schedule_invariants(m, n, bm, bn, group_m, wgs, xcd):
    npm, npn = osch.cdiv(m, bm), osch.cdiv(n, bn)
    nt = npm * npn
    g = min(wgs, nt)
    seen = {}
    for pos in range(nt):
        pm, pn, wg, rnd = oar.persistent_tile(pos, m, n, bm, bn, group_m, g, xcd)
        assert 0 <= pm < npm and 0 <= pn < npn
        assert (wg, rnd) == (pos % g, pos // g)                # work-group g takes positions g, g+G, ...
        seen[(pm, pn)] = pos
    assert len(seen) == nt                                      # every tile exactly once
    flags = sorted(oar.tile_flag_index(pm, pn, npn) for pm, pn in seen)
    assert flags == list(range(nt))                             # one flag per tile, row-major
    if xcd == 0:                                                # plain grouped order: row index runs fastest in a group
        assert oar.persistent_tile(0, m, n, bm, bn, group_m, g)[:2] == (0, 0)
        if npm > 1:
            assert oar.persistent_tile(1, m, n, bm, bn, group_m, g)[:2] == (1, 0)
    else:
        # the remap only permutes positions inside a round: the set of tiles of round r is unchanged
        for rnd in range(osch.cdiv(nt, g)):
            plain = {osch.grouped_order(t, npm, npn, group_m) for t in range(rnd * g, min(nt, (rnd + 1) * g))}
            mine = {oar.persistent_tile(p, m, n, bm, bn, group_m, g, xcd)[:2] for p in range(rnd * g, min(nt, (rnd + 1) * g))}
            assert plain == mine


def test_two_shot_ownership_is_a_partition():
    for world, nt in ((8, 1024), (3, 10), (4, 4), (1, 7)):
        owners = [oar.two_shot_owner(q, world) for q in range(nt)]
        assert set(owners) <= set(range(world))
        counts = np.bincount(owners, minlength=world)
        assert counts.sum() == nt and counts.max() - counts.min() <= 1      # every tile once, dealt evenly
        assert owners[:world] == list(range(world))[:nt]                    # in turn, starting with rank 0
