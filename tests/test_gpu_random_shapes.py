"""Seeded random problem shapes through the three dense operators, integer inputs, bit-exact against the
oracle: whatever tile, kernel or layout the library picks for a shape, the bits must not change."""
import numpy as np
import pytest
import torch

import synth
from oracle import ag_gemm as oag, gemm_rs as ors, gemm_ar as oar, formats

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, AgGemmRun, GemmRsRun, GemmArRun  # noqa: E402


def _shapes(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        world = int(rng.choice([1, 2, 3, 4, 8]))
        m_r = int(rng.integers(1, 700))
        n = 8 * int(rng.integers(1, 400))
        k = 8 * int(rng.integers(1, 60))
        out.append((world, m_r, n, k, int(rng.integers(0, world)), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("world,m_r,n,k,rank,kn", _shapes(11, 10))
def test_ag_gemm_random_shape(B, world, m_r, n, k, rank, kn):
    cfg = synth.CONFIGS[2].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=rank, seed=m_r)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    run = AgGemmRun(B, world, m_r, n, k)
    st = run([to_dev(s) for s in shards], to_dev(b if kn else nk(b)), rank, b_layout=B.B_KN if kn else B.B_NK)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(bits(run.c), formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32)))


@pytest.mark.parametrize("world,m_r,n,k,rank,kn", _shapes(12, 8))
def test_gemm_rs_random_shape(B, world, m_r, n, k, rank, kn):
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k, seed=n)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    # the peers' blocks for this rank: exact for integer inputs, so the oracle's partial is what a peer holds
    peers = [to_dev(formats.encode_bf16_rne(ors.partial(a_list[s][rank * m_r:(rank + 1) * m_r], b_list[s]).astype(np.float32)))
             for s in range(world)]
    run = GemmRsRun(B, world, cfg.m, n, k, chunks=1)
    b_dev = to_dev(b_list[rank] if kn else nk(b_list[rank]))
    st = run(to_dev(a_list[rank]), b_dev, peers, rank, b_layout=B.B_KN if kn else B.B_NK)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(bits(run.out), formats.encode_bf16_rne(ors.gemm_rs(a_list, b_list, rank).astype(np.float32)))


@pytest.mark.parametrize("world,m_r,n,k,rank,kn", _shapes(13, 8))
def test_gemm_ar_random_shape(B, world, m_r, n, k, rank, kn):
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k, seed=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    parts = [to_dev(oar.partial_bits(a, b)) for a, b in zip(a_list, b_list)]
    run = GemmArRun(B, world, cfg.m, n, k)
    b_dev = to_dev(b_list[rank] if kn else nk(b_list[rank]))
    peers = [None if s == rank else parts[s] for s in range(world)]
    st = run(to_dev(a_list[rank]), b_dev, peers if world > 1 else None, rank, b_layout=B.B_KN if kn else B.B_NK)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(bits(run.out), formats.encode_bf16_rne(oar.gemm_ar(a_list, b_list).astype(np.float32)))
