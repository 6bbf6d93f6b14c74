"""AllGather-GEMM on the GPU against the CPU oracle, through the C ABI."""
import itertools
import numpy as np
import pytest
import torch

import synth
from oracle import ag_gemm as oag, schedule as osch, formats, compare

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2   # max |err| <= 2e-2 * max |row| (stated for bf16 outputs with fp32 accumulation)


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, AgGemmRun  # noqa: E402


def _run(B, cfg, shards, b_kn, rank=None, order=None, want_schedule=False, kn=False, tuning=None):
    rank = cfg.rank if rank is None else rank
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    sh = [to_dev(s) for s in shards]
    bd = to_dev(b_kn if kn else nk(b_kn))     # kn: B handed over as it is stored, [k, n]
    sched = None
    if want_schedule:
        st, tc = B.tile_config(4 if kn else 0, cfg.m, cfg.n, cfg.k)
        sched = torch.full((4 * tc["ntiles"] * tc["splits"],), -1, dtype=torch.int32, device="cuda")
    st = run(sh, bd, rank, order=order, schedule=sched, b_layout=B.B_KN if kn else B.B_NK, tuning=tuning)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    return bits(run.c), bits(run.workspace), (None if sched is None else sched.cpu().numpy().reshape(-1, 4)), run


def _check(c_bits, ref64, tol=TOL_BF16):
    err = compare.max_row_rel_error(formats.decode_bf16(c_bits), ref64)
    assert err <= tol, err
    return err


def test_cfg1_world2_smoke(B):
    cfg = synth.CONFIGS[1]
    shards, b = synth.ag_gemm_inputs(cfg)
    c, ws, sched, _ = _run(B, cfg, shards, b, want_schedule=True)
    assert np.array_equal(ws, oag.gather(shards))          # the all-gather reproduces the input
    _check(c, oag.ag_gemm(shards, b))
    _check_schedule(B, cfg, cfg.rank, sched)


def _check_schedule(B, cfg, rank, sched, kn=False):
    st, tc = B.tile_config(4 if kn else 0, cfg.m, cfg.n, cfg.k)
    assert st == B.OK
    nt = tc["ntiles"]
    assert nt == osch.cdiv(cfg.m, tc["block_m"]) * osch.cdiv(cfg.n, tc["block_n"])
    want = []
    for wg in range(nt):
        pid = osch.xcd_remap(wg, nt, tc["num_xcd"], tc["per_xcd"]) if tc["num_xcd"] else wg
        # work-groups that share a tile's contraction share its record
        want += [osch.ag_tile(pid, cfg.m, cfg.n, tc["block_m"], tc["block_n"], tc["group_m"], rank, cfg.world)] * tc["splits"]
    assert np.array_equal(sched, np.asarray(want, dtype=np.int32))


@pytest.mark.parametrize("world,m_r,n,k", [
    (2, 128, 256, 256),      # one small tile row per shard
    (4, 200, 264, 328),      # ragged rows, columns and contraction tail (328 = 5*64 + 8)
    (8, 505, 3080, 200),     # 256x256 tiles with ragged edges on every side, 208 tiles
    (8, 505, 3080, 192),     # the same with a contraction of whole K tiles: operands staged straight into LDS
    (8, 505, 3080, 64),      # ... a single K tile
    (8, 505, 3080, 128),     # ... two K tiles
    (8, 250, 2056, 136),     # 128x128 tiles of the tile engine (too many for the decode kernel, too few 256x256 ones)
    (3, 64, 8, 8),           # minimum contraction and width
])
@pytest.mark.parametrize("kn", [False, True], ids=["b_nk", "b_kn"])
def test_integer_inputs_are_bit_exact(B, world, m_r, n, k, kn):
    # products and sums of small integers are exact in fp32, so the only rounding is the final
    # bf16 one: the GPU must match the oracle bit for bit, whatever the tile or lane layout
    cfg = synth.CONFIGS[2].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=world - 1)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    c, ws, sched, _ = _run(B, cfg, shards, b, want_schedule=True, kn=kn)
    want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    assert np.array_equal(ws, oag.gather(shards))
    assert np.array_equal(c, want)
    _check_schedule(B, cfg, cfg.rank, sched, kn=kn)


@pytest.mark.parametrize("world,m_r,n,k", [(4, 200, 264, 328), (8, 505, 3080, 456)])
@pytest.mark.parametrize("kn", [False, True], ids=["b_nk", "b_kn"])
def test_normal_inputs_within_tolerance(B, world, m_r, n, k, kn):
    cfg = synth.CONFIGS[2].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=1)
    shards, b = synth.ag_gemm_inputs(cfg)
    c, ws, _, _ = _run(B, cfg, shards, b, kn=kn)
    _check(c, oag.ag_gemm(shards, b))


def test_result_independent_of_rank_and_arrival_order(B):
    cfg = synth.CONFIGS[2].scaled(world=4, m_per_rank=192, n=384, k=512)
    shards, b = synth.ag_gemm_inputs(cfg)
    ref = None
    orders = [None, [3, 2, 1, 0], [1, 3, 0, 2]]
    for rank, order in itertools.product(range(cfg.world), orders):
        c, ws, _, _ = _run(B, cfg, shards, b, rank=rank, order=order)
        if ref is None:
            ref = c
            _check(c, oag.ag_gemm(shards, b))
        assert np.array_equal(c, ref), (rank, order)


def test_epoch_reuse_sees_fresh_data(B):
    # same buffers, new shard contents and a new epoch every call: a consumer that read a stale
    # copy of the workspace (left in a cache by the previous call) would fail here
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=256, n=2048, k=1024)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    _, b = synth.ag_gemm_inputs(cfg, integer=True)
    bd = to_dev(nk(b))
    for it in range(4):
        shards, _ = synth.ag_gemm_inputs(cfg.scaled(seed=it + 1), integer=True)
        sh = [to_dev(s) for s in shards]
        assert run(sh, bd, rank=it % cfg.world) == B.OK
        torch.cuda.synchronize()
        assert run.status.cpu().tolist()[0] == 0
        want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
        assert np.array_equal(bits(run.c), want), it
        assert run.signals.cpu().numpy()[:cfg.world].tolist() == [run.epoch] * cfg.world
        assert run.signals.cpu().numpy()[cfg.world:].tolist() == [0] * (run.signals.numel() - cfg.world)


def test_external_producer_and_timeout(B):
    cfg = synth.CONFIGS[2].scaled(world=4, m_per_rank=128, n=256, k=256)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    sh = [to_dev(s) for s in shards]
    bd = to_dev(nk(b))
    # (a) a separate publisher delivers the shards in a scrambled order with idle gaps; it is
    # enqueued first, on its own stream, and the consumer only waits
    side = torch.cuda.Stream()
    order = [2, 0, 3, 1]
    dst = [run.workspace[s * cfg.m_per_rank:(s + 1) * cfg.m_per_rank] for s in order]
    src = [sh[s] for s in order]
    nbytes = [cfg.m_per_rank * cfg.k * 2] * cfg.world
    st = B.publish_chunks(dst, src, nbytes, order, run.signals, run.epoch + 1, delay_cycles=20000, stream=side)
    assert st == B.OK
    assert run(None, bd, rank=1, flags=B.EXTERNAL_PRODUCER) == B.OK
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(bits(run.c), want)
    # (b) nobody raises the flags: with a tiny spin limit every wait gives up, the kernel ends
    # and reports the time-out instead of hanging
    assert run(None, bd, rank=0, flags=B.EXTERNAL_PRODUCER, tuning=B.tuning(spin_limit=64)) == B.OK
    torch.cuda.synchronize()
    s = run.status.cpu().tolist()
    assert s[0] == B.ERR_TIMEOUT and 0 <= s[1] < cfg.world
    # (c) the buffers stay usable afterwards
    run.status.zero_()
    assert run(sh, bd, rank=2) == B.OK
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0 and np.array_equal(bits(run.c), want)


def test_cfg2_full_size_every_element(B):
    cfg = synth.CONFIGS[2]
    shards, b = synth.ag_gemm_inputs(cfg)
    c, ws, sched, _ = _run(B, cfg, shards, b, want_schedule=True)
    assert np.array_equal(ws, oag.gather(shards))
    _check_schedule(B, cfg, cfg.rank, sched)
    cd = formats.decode_bf16(c)
    worst = 0.0
    for r0 in range(0, cfg.m, 1024):       # one shard of rows at a time keeps the fp64 copies small
        rows = np.arange(r0, r0 + 1024)
        worst = max(worst, compare.max_row_rel_error(cd[rows], oag.ag_gemm(shards, b, rows=rows)))
    assert worst <= TOL_BF16, worst


@pytest.mark.parametrize("world,nnodes,m_r,n,k", [
    (4, 2, 128, 256, 64),        # two nodes of two ranks, one small tile row per rank
    (8, 2, 200, 264, 72),        # tile rows shared between ranks and between the two nodes
    (8, 4, 505, 3080, 64),       # 256x256 tiles, four nodes
])
def test_tile_rows_follow_the_multi_node_order(B, world, nnodes, m_r, n, k):
    """With more than one node the kernel visits tile rows in the order of the paper's first swizzle
    listing (checked against the oracle through the schedule dump); the product does not change."""
    cfg = synth.CONFIGS[2].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    want_c = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    st, tc = B.tile_config(0, cfg.m, n, k)
    npm, npn = osch.cdiv(cfg.m, tc["block_m"]), osch.cdiv(n, tc["block_n"])
    for rank in (0, world // nnodes, world - 1):
        c, ws, sched, _ = _run(B, cfg, shards, b, rank=rank, want_schedule=True, tuning=B.tuning(num_nodes=nnodes))
        assert np.array_equal(c, want_c)
        want = []
        for wg in range(tc["ntiles"]):
            pid = osch.xcd_remap(wg, tc["ntiles"], tc["num_xcd"], tc["per_xcd"]) if tc["num_xcd"] else wg
            pm, pn = osch.grouped_order(pid, npm, npn, tc["group_m"])
            pm = osch.ag_swizzle_multinode(pm, cfg.m, rank, world, nnodes, tc["block_m"])
            row0 = pm * tc["block_m"]
            want += [(pm, pn, row0 // m_r, (min(row0 + tc["block_m"], cfg.m) - 1) // m_r)] * tc["splits"]
        assert np.array_equal(sched, np.asarray(want, dtype=np.int32))
        # the host evaluation of the schedule is the same list
        st, host = B.schedule_dump(0, cfg.m, n, k, world, rank, tuning=B.tuning(num_nodes=nnodes))
        assert st == B.OK and host == want


def test_multi_node_order_that_skips_rows_is_refused(B):
    # 37 rows per rank, four nodes, 128-row tiles: the listing's order is not a permutation of the
    # tile rows for rank 4; the library refuses instead of computing a partial product
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=37, n=128, k=64)
    st, order = B.tile_row_order(0, cfg.m, 128, 8, 4, 4)
    assert st == B.OK and sorted(order) != list(range(len(order)))
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    four = B.tuning(num_nodes=4)
    assert run([to_dev(s) for s in shards], to_dev(nk(b)), 4, tuning=four) == B.ERR_UNSUPPORTED
    assert run([to_dev(s) for s in shards], to_dev(nk(b)), 0, tuning=four) == B.OK      # rank 0's order is fine
    torch.cuda.synchronize()


@pytest.mark.parametrize("k", [8256, 12360, 16384, 16392])
@pytest.mark.parametrize("kn", [False, True], ids=["b_nk", "b_kn"])
def test_long_contraction_on_256_tiles_is_bit_exact(B, k, kn):
    """256 x 256 tiles over long contractions, small-integer inputs, both layouts of B, bit for bit: 8256 = 129 and
    16384 = 256 whole K tiles, 12360 and 16392 with a ragged last K tile (the loads' range test); [n, k] operands
    go straight into LDS, [k, n] operands through the register-staged loop."""
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=505, n=3080, k=k, rank=3)
    st, tc = B.tile_config(4 if kn else 0, cfg.m, cfg.n, cfg.k)
    assert (tc["block_m"], tc["block_n"], tc["direct_staging"]) == (256, 256, 0) if kn else (256, 224, 1)   # 16 x 14 tiles of 224 columns fill more of the last round than 16 x 13 of 256
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    c, ws, _, _ = _run(B, cfg, shards, b, kn=kn)
    want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    assert np.array_equal(c, want)


@pytest.mark.parametrize("k", [8, 40, 64, 72, 128, 136, 200, 320])
def test_short_contraction_on_256_tiles_is_bit_exact(B, k):
    """The direct-to-LDS loop of the 256-row tiles (256 and 224 columns) at the short end: one, two, three and five K tiles, with and without a
    ragged last one (fewer K tiles than the ring of operand pieces holds; past the end the last K tile is requested
    again), ragged tile rows and columns, small-integer inputs, bit for bit."""
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=505, n=3080 if k % 16 else 4096, k=k, rank=5)
    st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k)
    assert (tc["block_m"], tc["block_n"], tc["direct_staging"]) == (256, 224 if cfg.n == 3080 else 256, 1)   # both tile widths
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    c, ws, _, _ = _run(B, cfg, shards, b)
    want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    assert np.array_equal(c, want)


@pytest.mark.parametrize("k", [72, 192])
def test_192_column_tiles_are_bit_exact(B, k):
    """1376 columns (the LLaMA-7B share) go to 256 x 192 tiles: eight column blocks, the last one 32 columns wide."""
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=1024, n=1376, k=k, rank=2)
    st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k)
    assert (tc["block_m"], tc["block_n"], tc["ntiles"], tc["direct_staging"]) == (256, 192, 256, 1)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    c, ws, sched, _ = _run(B, cfg, shards, b, want_schedule=True)
    want = formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32))
    assert np.array_equal(c, want)
    _check_schedule(B, cfg, cfg.rank, sched)


def test_cfg2_full_size_other_rank_and_layout(B):
    """cfg 2 at full size from the view of rank 5, B stored [n, k] and [k, n]; every 16th row plus the
    rows around every shard boundary against the oracle, the schedule bit for bit."""
    cfg = synth.CONFIGS[2]
    shards, b = synth.ag_gemm_inputs(cfg)
    rows = np.unique(np.concatenate([np.arange(0, cfg.m, 16)] +
                                    [np.arange(s * cfg.m_per_rank - 2, s * cfg.m_per_rank + 2) % cfg.m for s in range(cfg.world)]))
    ref = oag.ag_gemm(shards, b, rows=rows)
    for kn in (False, True):
        c, ws, sched, _ = _run(B, cfg, shards, b, rank=5, want_schedule=True, kn=kn)
        _check_schedule(B, cfg, 5, sched, kn=kn)
        assert compare.max_row_rel_error(formats.decode_bf16(c[rows]), ref) <= TOL_BF16


def test_llama_405b_share_sampled(B):
    """The LLaMA-3.1-405B share of the paper's AllGather+GEMM shape table (M 8192, N 53248 / 8, K 16384)
    at full size: sampled rows of every shard against the oracle."""
    cfg = synth.CONFIGS[2].scaled(world=8, m_per_rank=1024, n=6656, k=16384, rank=2)
    shards, b = synth.ag_gemm_inputs(cfg)
    rows = np.unique(np.concatenate([np.arange(0, cfg.m, 41), np.arange(cfg.m - 3, cfg.m)]))
    c, ws, sched, _ = _run(B, cfg, shards, b, want_schedule=True)
    _check_schedule(B, cfg, cfg.rank, sched)
    assert compare.max_row_rel_error(formats.decode_bf16(c[rows]), oag.ag_gemm(shards, b, rows=rows)) <= TOL_BF16


def test_flags_preset_runs_the_gemm_alone(B):
    """DITRON_FLAGS_PRESET: the gathered operand is already in the workspace, nothing is copied and no
    flag is looked at (the signal words are all zero here and stay so)."""
    cfg = synth.CONFIGS[2].scaled(world=4, m_per_rank=200, n=264, k=328, rank=1)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    run.workspace.copy_(to_dev(oag.gather(shards)))
    assert run(None, to_dev(nk(b)), cfg.rank, flags=B.FLAGS_PRESET) == B.OK
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0 and not run.signals.any()
    assert np.array_equal(bits(run.c), formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32)))


@pytest.mark.parametrize("shape", [(4, 200, 264, 328), (8, 505, 3080, 192), (8, 16, 1024, 2048)])
def test_timing_dump_is_ordered_and_leaves_the_result_alone(B, shape):
    """DITRON_DUMP_TIMING: every GEMM work-group writes (start, wait entered, wait left, end), in that order in
    time; the product is what it is without the flag; the two dump flags exclude each other."""
    world, m_r, n, k = shape
    cfg = synth.CONFIGS[2].scaled(world=world, m_per_rank=m_r, n=n, k=k, rank=1)
    shards, b = synth.ag_gemm_inputs(cfg, integer=True)
    st, tc = B.tile_config(0, cfg.m, n, k)
    run = AgGemmRun(B, world, m_r, n, k)
    stamps = torch.zeros(4 * tc["ntiles"] * tc["splits"], dtype=torch.int32, device="cuda")
    sh, bd = [to_dev(s) for s in shards], to_dev(nk(b))
    assert run(sh, bd, 1, flags=B.EMULATE_PRODUCER | B.DUMP_TIMING | B.DUMP_SCHEDULE, schedule=stamps) == B.ERR_INVALID_ARG
    run.epoch += 1
    st = B.ag_gemm(sh, bd, B.B_NK, run.c, None, None, run.ws_raw, run.signals, run.status, stamps, None, m_r, n, k, world, 1,
                   B.BF16, run.epoch, B.EMULATE_PRODUCER | B.DUMP_TIMING)
    assert st == B.OK
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    assert np.array_equal(bits(run.c), formats.encode_bf16_rne(oag.ag_gemm(shards, b).astype(np.float32)))
    r = stamps.cpu().numpy().reshape(-1, 4).astype(np.int64)
    assert (r != 0).all()
    d = np.diff(r, axis=1) % (1 << 31)
    assert (d < (1 << 30)).all()                 # start <= wait entered <= wait left <= end (modulo the 31-bit wrap)
    assert ((r[:, 3] - r[:, 0]) % (1 << 31) < 100 * 1000 * 100).all()      # no work-group lives for 100 ms
