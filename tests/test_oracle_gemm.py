"""Pins for the floating-point oracles: brute-force loops on tiny inputs, closed forms,
special cases that reduce to a plain library GEMM, and the conservation laws that tie
AllGather-GEMM and GEMM-ReduceScatter to the unsharded product."""
import numpy as np
import pytest
import torch

import synth
from oracle import ag_gemm as oag, gemm_rs as ors, formats, compare


def _bf(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _brute_matmul(a, b):
    m, k = a.shape
    n = b.shape[1]
    c = [[0.0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            s = 0.0
            for t in range(k):
                s += float(a[i, t]) * float(b[t, j])
            c[i][j] = s
    return np.array(c)


def test_gather_places_shard_s_at_rows_s():
    shards = [np.full((3, 2), s, dtype=np.uint16) for s in range(4)]
    g = oag.gather(shards)
    assert g.shape == (12, 2)
    for s in range(4):
        assert (g[3 * s:3 * s + 3] == s).all()


def test_arrival_orders():
    assert oag.arrival_order(0, 2) == [0, 1]
    assert oag.arrival_order(5, 8) == [5, 6, 7, 0, 1, 2, 3, 4]
    # reduce-scatter: own block last, the rank just below arrives first
    assert ors.arrival_order(0, 8) == [7, 6, 5, 4, 3, 2, 1, 0]
    assert ors.arrival_order(3, 4) == [2, 1, 0, 3]
    for r in range(8):
        assert sorted(ors.arrival_order(r, 8)) == list(range(8))


@pytest.mark.parametrize("world,m_r,k,n", [(2, 2, 3, 2), (3, 1, 5, 4), (1, 4, 2, 3)])
def test_ag_gemm_brute_force_tiny(world, m_r, k, n):
    rng = np.random.default_rng(world * 100 + k)
    shards = [synth.normal_bf16(rng, (m_r, k)) for _ in range(world)]
    b = synth.normal_bf16(rng, (k, n))
    a_full = np.concatenate([formats.decode_bf16(s) for s in shards], axis=0)
    ref = _brute_matmul(a_full, formats.decode_bf16(b))
    got = oag.ag_gemm(shards, b)
    assert got.shape == (world * m_r, n)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_ag_gemm_closed_form_detects_transposition():
    # A[m,k] = m+1 for k == 0 else 0 ; B[k,n] = n+1 for k == 0 -> C[m,n] = (m+1)(n+1)
    world, m_r, k, n = 2, 3, 4, 5
    a = np.zeros((world * m_r, k), dtype=np.float32)
    a[:, 0] = np.arange(1, world * m_r + 1)
    b = np.zeros((k, n), dtype=np.float32)
    b[0, :] = np.arange(1, n + 1)
    shards = [_bf(a[s * m_r:(s + 1) * m_r]) for s in range(world)]
    got = oag.ag_gemm(shards, _bf(b))
    assert np.array_equal(got, np.outer(np.arange(1, 7), np.arange(1, 6)))


def test_ag_gemm_equals_library_gemm_cfg1():
    cfg = synth.CONFIGS[1]
    shards, b = synth.ag_gemm_inputs(cfg)
    got = oag.ag_gemm(shards, b)
    a_t = torch.cat([torch.from_numpy(s.view(np.int16).copy()).view(torch.bfloat16) for s in shards]).double()
    b_t = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).double()
    ref = (a_t @ b_t).numpy()
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    # rows= restricts without changing values
    rows = [0, 127, 128, 255]
    assert np.array_equal(oag.ag_gemm(shards, b, rows=rows), got[rows])


def test_ag_gemm_fp8_scales():
    cfg = synth.CONFIGS[5].scaled(m_per_rank=2, k=64, n=8, world=4)
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    unscaled = oag.ag_gemm(a, b, dtype="e4m3")
    ones = oag.ag_gemm(a, b, dtype="e4m3", a_scales=np.ones(4), b_scales=np.ones(8))
    assert np.array_equal(unscaled, ones)
    scaled = oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb)
    for m in range(8):
        for n in range(8):
            assert scaled[m, n] == pytest.approx(unscaled[m, n] * float(sa[m // 2]) * float(sb[n]), rel=1e-14)
    # the scaled product approximates the unquantised one
    x = np.concatenate([synth.rng_for(0, 5, 100 + s).standard_normal(size=(2, 64), dtype=np.float32)
                        for s in range(4)]).astype(np.float64)
    w = synth.rng_for(0, 5, 1).standard_normal(size=(64, 8), dtype=np.float32).astype(np.float64) / 8.0
    assert compare.max_row_rel_error(scaled, x @ w) < 0.15


@pytest.mark.parametrize("world,m,k,n", [(2, 4, 3, 2), (4, 8, 2, 3)])
def test_gemm_rs_brute_force_and_conservation(world, m, k, n):
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m // world, k=k, n=n)
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    # sum of the reduce-scatter shards == GEMM over the concatenated contraction dimension
    a_cat = np.concatenate([formats.decode_bf16(a) for a in a_list], axis=1)
    b_cat = np.concatenate([formats.decode_bf16(b) for b in b_list], axis=0)
    full = _brute_matmul(a_cat, b_cat)
    outs = [ors.gemm_rs(a_list, b_list, d) for d in range(world)]
    assert np.allclose(np.concatenate(outs, axis=0), full, rtol=1e-13, atol=1e-13)
    # stage oracle: partial of one rank
    p0 = ors.partial(a_list[0], b_list[0])
    assert np.allclose(p0, _brute_matmul(formats.decode_bf16(a_list[0]), formats.decode_bf16(b_list[0])),
                       rtol=1e-13, atol=1e-13)


def test_gemm_rs_world1_is_plain_gemm():
    cfg = synth.CONFIGS[3].scaled(world=1, m_per_rank=5, k=7, n=3)
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    assert np.array_equal(ors.gemm_rs(a_list, b_list, 0), ors.partial(a_list[0], b_list[0]))


def test_reduce_slots():
    rng = np.random.default_rng(5)
    slots = [synth.normal_bf16(rng, (6, 16)) for _ in range(8)]
    ref = sum(formats.decode_bf16(s) for s in slots)
    assert np.array_equal(ors.reduce_slots_f64(slots), ref)
    # integer slots: every order and precision gives the same bits
    islots = [synth.integer_bf16(rng, (6, 16), -3, 3) for _ in range(8)]
    exact = ors.reduce_slots_f64(islots)
    assert np.array_equal(formats.decode_bf16(ors.reduce_slots_f32_ordered(islots)), exact)
    # fp32-ordered result is within one bf16 ulp of the exact sum, and matches torch's
    # sequential fp32 adds
    got = ors.reduce_slots_f32_ordered(slots)
    t = [torch.from_numpy(s.view(np.int16).copy()).view(torch.bfloat16).float() for s in slots]
    acc = t[0].clone()
    for x in t[1:]:
        acc = acc + x
    tref = acc.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, tref)
    ulp = np.maximum(np.abs(ref), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(formats.decode_bf16(got) - ref) <= ulp)


def test_row_metric():
    ref = np.array([[1.0, -4.0], [0.0, 0.0], [2.0, 2.0]])
    got = np.array([[1.0, -4.4], [0.0, 0.0], [2.0, 2.0]])
    e = compare.row_rel_error(got, ref)
    assert e[0] == pytest.approx(0.1) and e[1] == 0 and e[2] == 0
    got[1, 0] = 1e-30
    assert compare.row_rel_error(got, ref)[1] == np.inf


def test_fused_scatter_rows_by_hand():
    # 2 ranks, 4 rows: rank 1's rows 0, 1 belong to rank 0 and land in its slot 1 (rows 2, 3); its rows 2, 3
    # are its own and land in its own slot 1 (rows 2, 3)
    assert [ors.fused_scatter_row(r, 1, 2, 4) for r in range(4)] == [(0, 2), (0, 3), (1, 2), (1, 3)]
    assert [ors.fused_scatter_row(r, 0, 2, 4) for r in range(4)] == [(0, 0), (0, 1), (1, 0), (1, 1)]
    # every destination buffer receives every one of its rows exactly once over all senders, and summing the
    # slots of a buffer gives the reduce-scatter result
    world, m, n = 4, 12, 3
    rng = np.random.default_rng(0)
    parts = [rng.integers(-4, 5, size=(m, n)).astype(np.float64) for _ in range(world)]
    bufs = [np.full((m, n), np.nan) for _ in range(world)]
    for s in range(world):
        for r in range(m):
            d, row = ors.fused_scatter_row(r, s, world, m)
            assert np.isnan(bufs[d][row]).all()
            bufs[d][row] = parts[s][r]
    m_r = m // world
    for d in range(world):
        assert not np.isnan(bufs[d]).any()
        assert np.array_equal(bufs[d].reshape(world, m_r, n).sum(axis=0), sum(p[d * m_r:(d + 1) * m_r] for p in parts))
