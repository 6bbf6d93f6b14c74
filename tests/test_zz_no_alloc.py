"""The entry point that allocates nothing (ditron_ag_gemm_static) against ditron_ag_gemm, through the C ABI:
two calls in a row on the library's one scratch array, the second smaller than the first, then an fp8
decode-shaped one; and the size limit."""
import numpy as np
import pytest
import torch

import synth
from oracle import ag_gemm as oag, formats

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, AgGemmRun  # noqa: E402


def _both(B, cfg, rank, integer):
    shards, b = synth.ag_gemm_inputs(cfg, integer=integer)
    sh, bd = [to_dev(s) for s in shards], to_dev(nk(b))
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    assert run(sh, bd, rank) == B.OK
    torch.cuda.synchronize()
    want = bits(run.c)
    c = torch.zeros_like(run.c)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    st = B.ag_gemm_static(sh, bd, B.B_NK, c, None, None, status, None, cfg.m_per_rank, cfg.n, cfg.k, cfg.world, rank, B.BF16)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert status.cpu().tolist()[0] == 0
    # same kernels, same tile order, same arithmetic: the two entry points agree bit for bit
    assert np.array_equal(bits(c), want)
    if integer:
        assert np.array_equal(want, formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32)))


def test_two_calls_in_a_row_second_smaller(B):
    big = synth.CONFIGS[2].scaled(world=8, m_per_rank=250, n=2056, k=1024)     # 128 x 128 tiles, 4 MB gathered
    small = synth.CONFIGS[2].scaled(world=4, m_per_rank=200, n=264, k=328)
    _both(B, big, rank=3, integer=True)
    _both(B, small, rank=1, integer=True)
    _both(B, big, rank=0, integer=False)


def test_fp8_decode_shape(B):
    cfg = synth.CONFIGS[5].scaled(n=1024, k=2048)
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    ad, bd, sad, sbd = [to_dev(x) for x in a], to_dev(nk(b)), to_dev(sa), to_dev(sb)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1)
    assert run(ad, bd, cfg.rank, dtype=B.FP8_E4M3, a_scales=sad, b_scales=sbd) == B.OK
    torch.cuda.synchronize()
    c = torch.zeros_like(run.c)
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    st = B.ag_gemm_static(ad, bd, B.B_NK, c, sad, sbd, status, None, cfg.m_per_rank, cfg.n, cfg.k, cfg.world, cfg.rank,
                          B.FP8_E4M3)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert status.cpu().tolist()[0] == 0 and np.array_equal(bits(c), bits(run.c))


def test_size_limit(B):
    fake = 0x1000
    st = B.ag_gemm_static([fake] * 8, fake, B.B_NK, fake, None, None, fake, None, 1024, 3584, 8192, 8, 0, B.BF16)
    assert st == B.ERR_WORKSPACE        # 128 MiB gathered operand: beyond the static array, nothing enqueued
    assert B.ag_gemm_static([fake] * 8, fake, B.B_NK, fake, None, None, fake, None, 0, 3584, 8192, 8, 0, B.BF16) == B.ERR_INVALID_ARG
