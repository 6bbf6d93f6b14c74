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


def _run(B, cfg, a, sa, b, sb, rank=None, order=None, want_schedule=False, variant=0):
    rank = cfg.rank if rank is None else rank
    tuning = B.tuning(decode_variant=variant)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1, tuning=tuning)
    sched = None
    st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k, B.FP8_E4M3, tuning)
    assert st == B.OK
    if want_schedule:
        sched = torch.full((4 * tc["ntiles"] * tc["splits"],), -1, dtype=torch.int32, device="cuda")
    st = run([to_dev(x) for x in a], to_dev(nk(b)), rank, order=order, schedule=sched, dtype=B.FP8_E4M3,
             a_scales=None if sa is None else to_dev(sa), b_scales=None if sb is None else to_dev(sb))
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(run.workspace.cpu().numpy(), oag.gather(a))
    if want_schedule:
        # one record per (tile, split of the contraction): the splits of a tile share the tile's record
        nt = tc["ntiles"]
        want = []
        for w in range(nt):
            pid = osch.xcd_remap(w, nt, tc["num_xcd"], tc["per_xcd"]) if tc["num_xcd"] else w
            want += [osch.ag_tile(pid, cfg.m, cfg.n, tc["block_m"], tc["block_n"], tc["group_m"], rank, cfg.world)] * tc["splits"]
        assert np.array_equal(sched.cpu().numpy().reshape(-1, 4), np.asarray(want, dtype=np.int32))
        st, host = B.schedule_dump(0, cfg.m, cfg.n, cfg.k, cfg.world, rank, B.FP8_E4M3, tuning=tuning)
        assert st == B.OK and host == want
        # the ticket counters of the split tiles are back at zero
        assert not run.signals.cpu().numpy()[cfg.world:].any()
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
@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4])
def test_fp8_integer_inputs_bit_exact(B, world, m_r, n, k, variant):
    cfg = synth.CONFIGS[5].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=world - 1)
    a, b = _integer_fp8(cfg, 3)
    got = _run(B, cfg, a, None, b, None, want_schedule=True, variant=variant)
    want = formats.encode_bf16_rne(oag.ag_gemm(a, b, dtype="e4m3").astype(np.float32))
    assert np.array_equal(got, want)
    if variant:
        return
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
    # every variant too: the split contraction is summed in split order whoever finishes last, so even
    # the variants that split agree with themselves bit for bit from run to run
    for rank, order, variant in [(0, None, 0), (3, None, 0), (1, [2, 0, 3, 1], 0), (2, [3, 2, 1, 0], 0)]:
        got = _run(B, cfg, a, sa, b, sb, rank=rank, order=order, variant=variant)
        if ref is None:
            ref = got
            err = compare.max_row_rel_error(formats.decode_bf16(got),
                                            oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb))
            assert err <= TOL_FP8
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4])
def test_cfg5_full_size(B, variant):
    cfg = synth.CONFIGS[5]
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    got = _run(B, cfg, a, sa, b, sb, want_schedule=True, variant=variant)
    ref = oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb)
    err = compare.max_row_rel_error(formats.decode_bf16(got), ref)
    assert err <= TOL_FP8, err
    assert err <= 1e-2          # what fp32 accumulation + one bf16 rounding should actually give


def test_epoch_in_memory_and_graph_replay(B):
    """DITRON_EPOCH_IN_MEMORY: the epoch lives in the last word of `signals` and the kernel advances it, so one
    recorded launch can be replayed.  Eager calls first, then a captured graph replayed several times with eager
    work and synchronisations in between; every result is compared with the call that takes its epoch as an
    argument."""
    cfg = synth.CONFIGS[5].scaled(world=8, m_per_rank=16, n=1024, k=2048, rank=3)
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    ref = _run(B, cfg, a, sa, b, sb)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1)
    xs, bd, sad, sbd = [to_dev(x) for x in a], to_dev(nk(b)), to_dev(sa), to_dev(sb)
    flags = B.EMULATE_PRODUCER | B.EPOCH_IN_MEMORY
    gathered = oag.gather(a)

    def check(calls_so_far):
        torch.cuda.synchronize()
        sig = run.signals.cpu().numpy()
        assert run.status.cpu().tolist()[0] == 0
        assert sig[-1] == calls_so_far and sig[-2] == 0              # the epoch advanced once, the counter is back at zero
        assert (sig[:cfg.world] == calls_so_far).all()               # every shard flag carries this call's epoch
        assert np.array_equal(bits(run.c), ref)
        assert np.array_equal(run.workspace.cpu().numpy(), gathered)

    for i in range(3):
        run.c.zero_()
        run.workspace.zero_()
        assert run(xs, bd, cfg.rank, flags=flags, dtype=B.FP8_E4M3, a_scales=sad, b_scales=sbd) == B.OK
        check(i + 1)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        try:
            st = run(xs, bd, cfg.rank, flags=flags, dtype=B.FP8_E4M3, a_scales=sad, b_scales=sbd, stream=side)
        finally:
            graph.capture_end()
    assert st == B.OK
    scratch = torch.zeros(1 << 20, device="cuda")
    for i in range(4):
        run.c.zero_()
        run.workspace.zero_()
        scratch.add_(1.0)                       # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        check(3 + i + 1)
    assert float(scratch[0]) == 4.0


def test_epoch_in_memory_is_refused_elsewhere(B):
    cfg = synth.CONFIGS[5].scaled(world=8, m_per_rank=16, n=1024, k=2048)
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1, tuning=B.tuning(decode_variant=1))
    st = run([to_dev(x) for x in a], to_dev(nk(b)), 0, flags=B.EMULATE_PRODUCER | B.EPOCH_IN_MEMORY, dtype=B.FP8_E4M3)
    assert st == B.ERR_UNSUPPORTED            # the 128 x 32 kernel takes its epoch as an argument only
    big = AgGemmRun(B, 2, 1024, 2048, 256)    # a bf16 problem of the tile engine
    x = [torch.zeros((1024, 256), dtype=torch.int16, device="cuda") for _ in range(2)]
    w = torch.zeros((2048, 256), dtype=torch.int16, device="cuda")
    assert big(x, w, 0, flags=B.EMULATE_PRODUCER | B.EPOCH_IN_MEMORY) == B.ERR_UNSUPPORTED
