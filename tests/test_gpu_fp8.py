"""fp8 (e4m3) AllGather-GEMM on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import ag_gemm as oag, schedule as osch, formats, compare

pytestmark = pytest.mark.gpu

TOL_FP8 = 5e-2     # stated bound for fp8 inputs; the accumulation itself is fp32


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, AgGemmRun  # noqa: E402


def _run(B, cfg, a, sa, b, sb, rank=None, order=None, want_schedule=False):
    rank = cfg.rank if rank is None else rank
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1)
    sched = None
    st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k, B.FP8_E4M3)
    assert st == B.OK
    if want_schedule:
        sched = torch.full((4 * tc["ntiles"],), -1, dtype=torch.int32, device="cuda")
    st = run([to_dev(x) for x in a], to_dev(nk(b)), rank, order=order, schedule=sched, dtype=B.FP8_E4M3,
             a_scales=None if sa is None else to_dev(sa), b_scales=None if sb is None else to_dev(sb))
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(run.workspace.cpu().numpy(), oag.gather(a))
    if want_schedule:
        nt = tc["ntiles"]
        want = [osch.ag_tile(osch.xcd_remap(w, nt, tc["num_xcd"], tc["per_xcd"]), cfg.m, cfg.n, tc["block_m"],
                             tc["block_n"], tc["group_m"], rank, cfg.world) for w in range(nt)]
        assert np.array_equal(sched.cpu().numpy().reshape(-1, 4), np.asarray(want, dtype=np.int32))
    return bits(run.c)


def _integer_fp8(cfg, seed):
    rng = synth.rng_for(seed, cfg.cfg_id, 9)
    a = [synth.quantize_e4m3(rng.integers(-2, 3, size=(cfg.m_per_rank, cfg.k)).astype(np.float64), 1.0)
         for _ in range(cfg.world)]
    b = synth.quantize_e4m3(rng.integers(-2, 3, size=(cfg.k, cfg.n)).astype(np.float64), 1.0)
    return a, b


@pytest.mark.parametrize("world,m_r,n,k", [
    (8, 16, 256, 256),       # decode-like: one row tile waits for all shards
    (8, 16, 8192, 1024),
    (4, 50, 264, 400),       # ragged rows / columns, contraction tail of 16
    (4, 100, 40, 16),        # several row tiles, minimum contraction, fewer K tiles than ring slots
    (2, 8, 8, 4096),
    (4, 40, 1000, 2192),     # odd number of K tiles plus a contraction tail of 16
    (8, 256, 2048, 384),     # many tiles
    (2, 640, 2560, 512),     # several row tiles per shard
])
def test_fp8_integer_inputs_bit_exact(B, world, m_r, n, k):
    cfg = synth.CONFIGS[5].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=world - 1)
    a, b = _integer_fp8(cfg, 3)
    got = _run(B, cfg, a, None, b, None, want_schedule=True)
    want = formats.encode_bf16_rne(oag.ag_gemm(a, b, dtype="e4m3").astype(np.float32))
    assert np.array_equal(got, want)
    # power-of-two scales keep everything exact as well
    sa = np.array([2.0 ** (s % 3 - 1) for s in range(world)], dtype=np.float32)
    sb = np.array([2.0 ** (j % 4 - 2) for j in range(n)], dtype=np.float32)
    got = _run(B, cfg, a, sa, b, sb, rank=0)
    want = formats.encode_bf16_rne(oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb).astype(np.float32))
    assert np.array_equal(got, want)


def test_fp8_rank_and_order_independent(B):
    cfg = synth.CONFIGS[5].scaled(world=4, m_per_rank=48, n=512, k=768)
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    ref = None
    for rank, order in [(0, None), (3, None), (1, [2, 0, 3, 1]), (2, [3, 2, 1, 0])]:
        got = _run(B, cfg, a, sa, b, sb, rank=rank, order=order)
        if ref is None:
            ref = got
            err = compare.max_row_rel_error(formats.decode_bf16(got),
                                            oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb))
            assert err <= TOL_FP8
        assert np.array_equal(got, ref)


def test_cfg5_full_size(B):
    cfg = synth.CONFIGS[5]
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    got = _run(B, cfg, a, sa, b, sb, want_schedule=True)
    ref = oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb)
    err = compare.max_row_rel_error(formats.decode_bf16(got), ref)
    assert err <= TOL_FP8, err
    assert err <= 1e-2          # what fp32 accumulation + one bf16 rounding should actually give
