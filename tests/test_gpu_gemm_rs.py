"""GEMM-ReduceScatter on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import gemm_rs as ors, schedule as osch, formats, compare

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, GemmRsRun  # noqa: E402


def _ok(B, st, run):
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0


@pytest.mark.parametrize("world,rows,n,chunks,gated", [
    (8, 64, 256, 1, False), (8, 96, 1000 * 8, 4, True), (4, 33, 40, 1, True), (3, 10, 8, 2, False),
    (1, 5, 16, 1, True), (2, 128, 4096, 8, True)])
def test_reduce_slots_exact(B, world, rows, n, chunks, gated):
    rng = synth.rng_for(7, world, rows)
    slots = [synth.normal_bf16(rng, (rows, n), std=3.0) for _ in range(world)]
    sd = [to_dev(s) for s in slots]
    out = torch.zeros((rows, n), dtype=torch.int16, device="cuda")
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    sig = torch.full((world * chunks,), 5, dtype=torch.int32, device="cuda") if gated else None
    st = B.reduce_slots(sd, out, sig, status, rows, n, world, chunks, 5)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert status.cpu().tolist()[0] == 0
    got = bits(out)
    # specified arithmetic: fp32 adds in slot order, one rounding -> identical bits
    assert np.array_equal(got, ors.reduce_slots_f32_ordered(slots))
    # and within one bf16 ulp of the exact sum
    exact = ors.reduce_slots_f64(slots)
    ulp = np.maximum(np.abs(exact), 2.0 ** -126) * 2.0 ** -7
    assert np.all(np.abs(formats.decode_bf16(got) - exact) <= ulp)


def _all_partials(B, cfg, a_list, b_list):
    """Every emulated rank's full partial product, computed by the library's own GEMM (this
    is what each peer would hold); returns device tensors [m, n]."""
    run = GemmRsRun(B, cfg.world, cfg.m, cfg.n, cfg.k)
    zero = torch.zeros((cfg.m_per_rank, cfg.n), dtype=torch.int16, device="cuda")
    parts = []
    for s in range(cfg.world):
        st = run(to_dev(a_list[s]), to_dev(nk(b_list[s])), [zero] * cfg.world, s)
        _ok(B, st, run)
        parts.append(run.gemm_out.clone())
    return parts


def _check_schedule(B, cfg, rank, sched):
    st, tc = B.tile_config(1, cfg.m, cfg.n, cfg.k)
    nt = tc["ntiles"]
    want = []
    for wg in range(nt):
        pid = osch.xcd_remap(wg, nt, tc["num_xcd"], tc["per_xcd"]) if tc["num_xcd"] else wg
        want.append(osch.rs_tile(pid, cfg.m, cfg.n, tc["block_m"], tc["block_n"], tc["group_m"], rank, cfg.world))
    assert np.array_equal(sched, np.asarray(want, dtype=np.int32))


@pytest.mark.parametrize("world,m_r,n,k,chunks,integer", [
    (4, 128, 256, 64, 1, True),
    (4, 100, 264, 72, 2, True),       # segments that straddle tiles, ragged everything
    (8, 505, 3080, 200, 5, True),     # 256x256 tiles, ragged edges
    (8, 505, 3080, 192, 5, True),     # the same with whole K tiles: operands staged straight into LDS
    (8, 505, 3080, 64, 5, True),      # ... a single K tile
    (8, 505, 3080, 1096, 5, True),    # ... 17 K tiles and a ragged 18th: several turns of the ring of operand pieces
    (2, 192, 384, 512, 3, False),
    (1, 256, 256, 128, 1, True),      # world 1: plain GEMM
])
@pytest.mark.parametrize("kn", [False, True], ids=["b_nk", "b_kn"])
def test_gemm_rs_end_to_end(B, world, m_r, n, k, chunks, integer, kn):
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=integer)
    parts = _all_partials(B, cfg, a_list, b_list)
    for s in (0, world - 1):     # stage oracle: the partial product itself
        err = compare.max_row_rel_error(formats.decode_bf16(bits(parts[s])), ors.partial(a_list[s], b_list[s]))
        assert err <= TOL_BF16
    run = GemmRsRun(B, world, cfg.m, n, k, chunks)
    st, tc = B.tile_config(1, cfg.m, n, k)
    for d in range(world):
        peers = [parts[s][d * m_r:(d + 1) * m_r] for s in range(world)]
        sched = torch.full((4 * tc["ntiles"],), -1, dtype=torch.int32, device="cuda")
        order = None if d % 2 == 0 else [s for s in range(world) if s != d]     # also a non-ring delivery
        b_dev = to_dev(b_list[d] if kn else nk(b_list[d]))      # kn: B handed over as it is stored, [k, n]
        st = run(to_dev(a_list[d]), b_dev, peers, d, order=order, schedule=sched, b_layout=B.B_KN if kn else B.B_NK)
        _ok(B, st, run)
        ref = ors.gemm_rs(a_list, b_list, d)
        got = bits(run.out)
        if integer:
            assert np.array_equal(got, formats.encode_bf16_rne(ref.astype(np.float32))), d
        else:
            assert compare.max_row_rel_error(formats.decode_bf16(got), ref) <= TOL_BF16
        _check_schedule(B, cfg, d, sched.cpu().numpy().reshape(-1, 4))
        sig = run.signals.cpu().numpy()
        assert sig[:world].tolist() == [run.epoch] * world            # every segment flag raised
        assert sig[world:2 * world].tolist() == [0] * world            # counters left at zero
        arr = sig[2 * world:2 * world + world * chunks].reshape(world, chunks)
        for s in range(world):
            if s != d:                                                  # every peer chunk was flagged
                assert arr[s].tolist() == [run.epoch] * chunks
        # the scatter buffer holds exactly what the peers sent
        for s in range(world):
            if s != d:
                assert torch.equal(run.scatter[s], peers[s])


def test_cfg3_full_size(B):
    cfg = synth.CONFIGS[3]
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    parts = _all_partials(B, cfg, a_list, b_list)
    d, m_r = cfg.rank, cfg.m_per_rank
    run = GemmRsRun(B, cfg.world, cfg.m, cfg.n, cfg.k, chunks=4)
    peers = [parts[s][d * m_r:(d + 1) * m_r] for s in range(cfg.world)]
    st = run(to_dev(a_list[d]), to_dev(nk(b_list[d])), peers, d)
    _ok(B, st, run)
    ref = ors.gemm_rs(a_list, b_list, d)
    assert compare.max_row_rel_error(formats.decode_bf16(bits(run.out)), ref) <= TOL_BF16
    # the reduction in isolation on the actual slot contents: bit-exact to the specified arithmetic
    slots = [bits(parts[s][d * m_r:(d + 1) * m_r]) for s in range(cfg.world)]
    assert np.array_equal(bits(run.out), ors.reduce_slots_f32_ordered(slots))
    # sampled rows of the partial product
    rows = np.arange(0, cfg.m, 61)
    pref = formats.decode_bf16(a_list[d][rows]) @ formats.decode_bf16(b_list[d])
    assert compare.max_row_rel_error(formats.decode_bf16(bits(run.gemm_out)[rows]), pref) <= TOL_BF16


@pytest.mark.parametrize("world,nnodes,m_r,n,k,chunks", [
    (4, 2, 128, 256, 64, 1),
    (8, 2, 200, 264, 72, 2),       # tile rows shared between segments and between the two nodes
])
def test_gemm_rs_multi_node_order(B, world, nnodes, m_r, n, k, chunks):
    """Scatter order across nodes (the paper's second swizzle listing): next node first, own segment
    last; the reduced output and the segment flags are what they are with one node."""
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    parts = _all_partials(B, cfg, a_list, b_list)
    run = GemmRsRun(B, world, cfg.m, n, k, chunks)
    st, tc = B.tile_config(1, cfg.m, n, k)
    npm, npn = osch.cdiv(cfg.m, tc["block_m"]), osch.cdiv(n, tc["block_n"])
    for d in (0, world // nnodes, world - 1):
        peers = [parts[s][d * m_r:(d + 1) * m_r] for s in range(world)]
        sched = torch.full((4 * tc["ntiles"],), -1, dtype=torch.int32, device="cuda")
        st = run(to_dev(a_list[d]), to_dev(nk(b_list[d])), peers, d, schedule=sched, tuning=B.tuning(num_nodes=nnodes))
        _ok(B, st, run)
        assert np.array_equal(bits(run.out), formats.encode_bf16_rne(ors.gemm_rs(a_list, b_list, d).astype(np.float32)))
        want = []
        for wg in range(tc["ntiles"]):
            pid = osch.xcd_remap(wg, tc["ntiles"], tc["num_xcd"], tc["per_xcd"]) if tc["num_xcd"] else wg
            pm, pn = osch.grouped_order(pid, npm, npn, tc["group_m"])
            pm = osch.rs_swizzle_multinode(pm, cfg.m, d, world, nnodes, tc["block_m"])
            want.append((pm, pn, (pm * tc["block_m"]) // m_r, (min((pm + 1) * tc["block_m"], cfg.m) - 1) // m_r))
        assert np.array_equal(sched.cpu().numpy().reshape(-1, 4), np.asarray(want, dtype=np.int32))
        sig = run.signals.cpu().numpy()
        assert sig[:world].tolist() == [run.epoch] * world


@pytest.mark.parametrize("world,m_r,n,k,chunks,integer", [
    (4, 128, 256, 64, 1, True),
    (4, 100, 264, 72, 2, True),       # tiles that straddle two or three segments, ragged everything
    (8, 505, 3080, 200, 5, True),     # 256x256 tiles
    (2, 192, 384, 512, 3, False),
    (1, 256, 256, 128, 1, True),
])
def test_gemm_rs_fused_scatter(B, world, m_r, n, k, chunks, integer):
    """The FUSE_SCATTER branch of the producer listing: segment d of the partial goes straight to slot `rank`
    of rank d's buffer (rows rank*M_r + m % M_r); the reduced output is what the unfused path gives."""
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=integer)
    parts = _all_partials(B, cfg, a_list, b_list)
    signals = torch.zeros(B.signal_words(world, chunks), dtype=torch.int32, device="cuda")
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    out = torch.zeros((m_r, n), dtype=torch.int16, device="cuda")
    for epoch, d in enumerate(sorted({0, world - 1}), start=1):
        dsts = [torch.full((world, m_r, n), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(world)]
        peers = [parts[s][d * m_r:(d + 1) * m_r] for s in range(world)]
        st = B.gemm_rs_fuse_scatter(to_dev(a_list[d]), to_dev(nk(b_list[d])), B.B_NK, dsts, peers, out, signals, status,
                                    None, None, cfg.m, n, k, world, d, chunks, epoch, B.EMULATE_PRODUCER)
        assert st == B.OK, B.status_string(st)
        torch.cuda.synchronize()
        assert status.cpu().tolist()[0] == 0
        own = bits(parts[d])                       # this rank's partial as the unfused GEMM writes it
        for t in range(world):
            buf = bits(dsts[t])
            # slot d of every rank's buffer holds segment t of this rank's partial, at the rows the listing gives
            for r in (t * m_r, t * m_r + m_r // 2, (t + 1) * m_r - 1):
                dest, row = ors.fused_scatter_row(r, d, world, cfg.m)
                assert dest == t and np.array_equal(buf.reshape(world * m_r, n)[row], own[r])
            assert np.array_equal(buf[d], own[t * m_r:(t + 1) * m_r])
            for s in range(world):
                if s == d:
                    continue
                if t == d:
                    assert torch.equal(dsts[t][s], peers[s])       # the peers' blocks arrived in the local buffer
                else:
                    assert (buf[s] == 0x7FC0).all()                # nothing else of a remote buffer is touched
        ref = ors.gemm_rs(a_list, b_list, d)
        got = bits(out)
        if integer:
            assert np.array_equal(got, formats.encode_bf16_rne(ref.astype(np.float32))), d
        else:
            assert compare.max_row_rel_error(formats.decode_bf16(got), ref) <= TOL_BF16
        assert np.array_equal(got, ors.reduce_slots_f32_ordered([bits(dsts[d][s]) for s in range(world)]))


def test_flags_preset_skips_the_peers(B):
    """DITRON_FLAGS_PRESET: the peers' blocks are already in the scatter buffer; only the GEMM's own
    segment flag gates the reduction and no arrival flag is touched."""
    cfg = synth.CONFIGS[3].scaled(world=4, m_per_rank=100, n=264, k=72)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    parts = _all_partials(B, cfg, a_list, b_list)
    d, m_r, world = 2, cfg.m_per_rank, cfg.world
    run = GemmRsRun(B, world, cfg.m, cfg.n, cfg.k, chunks=2)
    for s in range(world):
        if s != d:
            run.scatter[s].copy_(parts[s][d * m_r:(d + 1) * m_r])
    st = run(to_dev(a_list[d]), to_dev(nk(b_list[d])), None, d, flags=B.FLAGS_PRESET)
    _ok(B, st, run)
    assert np.array_equal(bits(run.out), formats.encode_bf16_rne(ors.gemm_rs(a_list, b_list, d).astype(np.float32)))
    sig = run.signals.cpu().numpy()
    assert sig[:world].tolist() == [run.epoch] * world and not sig[world:].any()


def test_llama_405b_share_sampled(B):
    """The LLaMA-3.1-405B share of the paper's GEMM+ReduceScatter shape table (M 8192, N 16384, K 53248 / 8)
    at full size: sampled rows of the partial product against the oracle, the reduction bit for bit
    against the ordered fp32 sum of the blocks that were in the slots."""
    cfg = synth.CONFIGS[3].scaled(world=8, m_per_rank=1024, n=16384, k=6656, rank=6)
    d, m_r = cfg.rank, cfg.m_per_rank
    rng = synth.rng_for(11, d, 405)
    a = synth.normal_bf16(rng, (cfg.m, cfg.k), std=1.0)
    b = synth.normal_bf16(rng, (cfg.k, cfg.n), std=cfg.k ** -0.5)
    peers_np = [synth.normal_bf16(rng, (m_r, cfg.n), std=1.0) for _ in range(cfg.world)]
    run = GemmRsRun(B, cfg.world, cfg.m, cfg.n, cfg.k, chunks=4)
    st, tc = B.tile_config(1, cfg.m, cfg.n, cfg.k)
    assert tc["block_m"] == 256
    sched = torch.full((4 * tc["ntiles"],), -1, dtype=torch.int32, device="cuda")
    st = run(to_dev(a), to_dev(nk(b)), [to_dev(p) for p in peers_np], d, schedule=sched)
    _ok(B, st, run)
    _check_schedule(B, cfg, d, sched.cpu().numpy().reshape(-1, 4))
    rows = np.unique(np.concatenate([np.arange(0, cfg.m, 53), np.arange(d * m_r, d * m_r + 4)]))
    pref = formats.decode_bf16(a[rows]) @ formats.decode_bf16(b)
    gemm_out = bits(run.gemm_out)
    assert compare.max_row_rel_error(formats.decode_bf16(gemm_out[rows]), pref) <= TOL_BF16
    slots = [gemm_out[d * m_r:(d + 1) * m_r] if s == d else peers_np[s] for s in range(cfg.world)]
    assert np.array_equal(bits(run.out), ors.reduce_slots_f32_ordered(slots))
