"""GEMM + AllReduce on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import gemm_ar as oar, schedule as osch, formats, compare

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2   # max |err| <= 2e-2 * max |row| (bf16 outputs, fp32 accumulation)


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, nk, GemmArRun  # noqa: E402


def _ok(B, st, run):
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0


def _check_schedule(run, cfg, sched):
    tc = run.tc
    nt = run.ntiles
    want = [oar.tile_at_position(pos, cfg.m, cfg.n, tc["block_m"], tc["block_n"], tc["group_m"], tc["num_xcd"],
                                 tc["per_xcd"]) for pos in range(nt)]
    assert np.array_equal(sched[:, :2], np.asarray(want, dtype=np.int32))
    # where the tiles sit in the launch (consumers in between not counted as tiles): in order, and on the
    # chiplet the remap assumes
    grid = sched[:, 2]
    assert (np.diff(grid) > 0).all()
    assert ((grid - np.arange(nt)) % 8 == 0).all()


@pytest.mark.parametrize("kn", [False, True], ids=["b_nk", "b_kn"])
@pytest.mark.parametrize("world,m_r,n,k,integer", [
    (4, 32, 256, 64, True),        # one tile row
    (4, 100, 264, 72, True),       # ragged rows, columns and contraction tail
    (8, 505, 3080, 200, True),     # 256x256 tiles with ragged edges, a single round: all tiles, then the consumers
    (8, 505, 3080, 192, True),     # the same with whole K tiles: operands staged straight into LDS
    (8, 505, 3080, 1096, True),    # 17 K tiles and a ragged 18th: several turns of the ring of operand pieces
    (8, 315, 2600, 64, True),      # 420 tiles of 128x128: more than one round, consumers behind the first one
    (2, 192, 384, 512, False),
    (1, 256, 256, 128, True),      # world 1: the all-reduce is a copy of the partial
    (3, 40, 8, 8, True),           # minimum contraction and width, rows not a multiple of anything
])
def test_gemm_ar_end_to_end(B, world, m_r, n, k, integer, kn):
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=integer)
    parts = [oar.partial_bits(a, b) for a, b in zip(a_list, b_list)]     # what each peer publishes
    parts_dev = [to_dev(p) for p in parts]
    ref = oar.gemm_ar(a_list, b_list)
    run = GemmArRun(B, world, cfg.m, n, k)
    for d in sorted({0, world - 1}):
        sched = torch.full((4 * run.ntiles,), -1, dtype=torch.int32, device="cuda")
        b_dev = to_dev(b_list[d] if kn else nk(b_list[d]))
        peers = [None if s == d else parts_dev[s] for s in range(world)]
        run.out.fill_(0x7FC0)
        st = run(to_dev(a_list[d]), b_dev, peers if world > 1 else None, d, schedule=sched,
                 b_layout=B.B_KN if kn else B.B_NK)
        _ok(B, st, run)
        own = bits(run.gemm_out)
        got = bits(run.out)
        if integer:
            assert np.array_equal(own, parts[d]), d
            assert np.array_equal(got, formats.encode_bf16_rne(ref.astype(np.float32))), d
        else:
            pref = formats.decode_bf16(a_list[d]) @ formats.decode_bf16(b_list[d])
            assert compare.max_row_rel_error(formats.decode_bf16(own), pref) <= TOL_BF16
            assert compare.max_row_rel_error(formats.decode_bf16(got), ref) <= TOL_BF16
        # the consumer on what was actually published: bit-exact to the specified arithmetic
        published = [own if s == d else parts[s] for s in range(world)]
        assert np.array_equal(got, oar.allreduce_partials_f32_ordered(published)), d
        _check_schedule(run, cfg, sched.cpu().numpy().reshape(-1, 4))
        sig = run.signals.cpu().numpy()
        assert not sig[:2 * world].any()                                # the queue counters are back at zero
        flags = sig[2 * world:2 * world + world * run.ntiles]
        assert flags.tolist() == [run.epoch] * (world * run.ntiles)     # every tile of every rank was announced


def test_external_producer_and_timeout(B):
    world, m, n, k, d = 4, 256, 256, 64, 1
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m // world, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    parts = [oar.partial_bits(a, b) for a, b in zip(a_list, b_list)]
    want = formats.encode_bf16_rne(oar.gemm_ar(a_list, b_list).astype(np.float32))
    run = GemmArRun(B, world, m, n, k)
    bm, bn = run.tc["block_m"], run.tc["block_n"]
    npm, npn = m // bm, n // bn
    assert (npm, npn) == (2, 2)
    src = [to_dev(p) for p in parts]
    landing = [torch.zeros((m, n), dtype=torch.int16, device="cuda") for _ in range(world)]   # the peers' buffers
    a_dev, b_dev = to_dev(a_list[d]), to_dev(nk(b_list[d]))
    # (a) a separate publisher fills the peers' buffers tile row by tile row, in a scrambled order and
    # with idle gaps, raising each tile's flag after its data; the consumer only waits
    dst, srcs, nbytes, fidx = [], [], [], []
    for s in (3, 0, 2):
        for pm in (1, 0):
            for pn in range(npn):
                rows = slice(pm * bm, (pm + 1) * bm)
                dst.append(landing[s][rows] if pn == 0 else None)
                srcs.append(src[s][rows] if pn == 0 else None)
                nbytes.append(bm * n * 2 if pn == 0 else 0)       # the second tile of the row rides on the same copy
                fidx.append(run.flag_index(s, pm, pn))
    side = torch.cuda.Stream()
    assert B.publish_chunks(dst, srcs, nbytes, fidx, run.signals, run.epoch + 1, delay_cycles=20000, stream=side) == B.OK
    peers = [None if s == d else landing[s] for s in range(world)]
    st = run(a_dev, b_dev, peers, d, flags=B.EXTERNAL_PRODUCER)
    _ok(B, st, run)
    assert np.array_equal(bits(run.out), want)
    # (b) nobody raises the peers' flags: with a tiny spin limit every wait gives up, the kernel ends and
    # reports the time-out instead of hanging, and leaves the queue counters at zero
    assert run(a_dev, b_dev, peers, d, flags=B.EXTERNAL_PRODUCER, tuning=B.tuning(spin_limit=64)) == B.OK
    torch.cuda.synchronize()
    s = run.status.cpu().tolist()
    assert s[0] == B.ERR_TIMEOUT and 0 <= s[1] < run.ntiles
    assert run.signals.cpu().numpy()[:2].tolist() == [0, 0]
    # (c) the buffers stay usable afterwards
    run.status.zero_()
    st = run(a_dev, b_dev, [None if s == d else src[s] for s in range(world)], d)
    _ok(B, st, run)
    assert np.array_equal(bits(run.out), want)


def test_table_shape_full_size(B):
    """Shape 3 of the paper's GEMM + AllReduce table at tensor parallel 8: M 8192, N 8192, K 28672 / 8.
    The peers' partials are made by the same GEMM (world 1 calls), as on a real node."""
    cfg = synth.CONFIGS[3]
    assert (cfg.m, cfg.n, cfg.k, cfg.world) == (8192, 8192, 3584, 8)
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    d = cfg.rank
    solo = GemmArRun(B, 1, cfg.m, cfg.n, cfg.k)
    parts_dev = []
    for s in range(cfg.world):
        if s == d:
            parts_dev.append(None)
            continue
        st = solo(to_dev(a_list[s]), to_dev(nk(b_list[s])), None, 0)
        _ok(B, st, solo)
        parts_dev.append(solo.gemm_out.clone())
    run = GemmArRun(B, cfg.world, cfg.m, cfg.n, cfg.k)
    st = run(to_dev(a_list[d]), to_dev(nk(b_list[d])), parts_dev, d)
    _ok(B, st, run)
    got = bits(run.out)
    published = [bits(run.gemm_out) if s == d else bits(parts_dev[s]) for s in range(cfg.world)]
    assert np.array_equal(got, oar.allreduce_partials_f32_ordered(published))
    rows = np.arange(0, cfg.m, 67)       # sampled rows, every tile row and column, against the definition
    ref = oar.gemm_ar(a_list, b_list, rows=rows)
    assert compare.max_row_rel_error(formats.decode_bf16(got[rows]), ref) <= TOL_BF16


@pytest.mark.parametrize("world,m_r,n,k,integer", [
    (4, 32, 256, 64, True),
    (4, 100, 264, 72, True),       # ragged edges, 12 tiles
    (8, 505, 3080, 200, True),     # 256x256 tiles, 208 of them
    (8, 315, 2600, 64, True),      # 420 tiles: more than one round
    (3, 128, 384, 128, False),     # a world that does not divide the tile count
    (1, 256, 256, 128, True),
])
def test_gemm_ar_two_shot(B, world, m_r, n, k, integer):
    """The broadcast branch of the consumer listing: the rank reduces the tiles it owns and stores them
    into every rank's output; the rest of its own output arrives from the owners."""
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=integer)
    parts = [oar.partial_bits(a, b) for a, b in zip(a_list, b_list)]
    parts_dev = [to_dev(p) for p in parts]
    run = GemmArRun(B, world, cfg.m, n, k)
    bm, bn = run.tc["block_m"], run.tc["block_n"]
    for d in sorted({0, world - 1}):
        sched = torch.full((4 * run.ntiles,), -1, dtype=torch.int32, device="cuda")
        outs = [torch.full((cfg.m, n), 0x7FC0, dtype=torch.int16, device="cuda") for _ in range(world)]
        peers = [None if s == d else parts_dev[s] for s in range(world)]
        run.epoch += 1
        a_dev, b_dev = to_dev(a_list[d]), to_dev(nk(b_list[d]))
        # what the peers broadcast: the all-reduce of what every rank publishes (this rank's own partial comes
        # from a first, one-shot call, as its peers would see it)
        st = run(a_dev, b_dev, peers if world > 1 else None, d)
        _ok(B, st, run)
        published = [bits(run.gemm_out) if s == d else parts[s] for s in range(world)]
        full = oar.allreduce_partials_f32_ordered(published)
        reduced = [None if s == d else to_dev(full) for s in range(world)]
        run.epoch += 1
        st = B.gemm_ar_two_shot(a_dev, b_dev, B.B_NK, run.gemm_out, peers if world > 1 else None, outs,
                                reduced if world > 1 else None, run.signals, run.status, sched, cfg.m, n, k, world, d,
                                run.epoch, B.EMULATE_PRODUCER | B.DUMP_SCHEDULE)
        _ok(B, st, run)
        assert np.array_equal(bits(outs[d]), full)                      # own output: complete
        rec = sched.cpu().numpy().reshape(-1, 4)
        _check_schedule(run, cfg, rec)
        for t in range(world):
            if t == d:
                continue
            buf = bits(outs[t])
            for q in range(run.ntiles):                                  # a peer's output: exactly the tiles this rank owns
                pm, pn = rec[q, 0], rec[q, 1]
                blk = (slice(pm * bm, min((pm + 1) * bm, cfg.m)), slice(pn * bn, min((pn + 1) * bn, n)))
                if oar.two_shot_owner(q, world) == d:
                    assert np.array_equal(buf[blk], full[blk]), (t, q)
                else:
                    assert (buf[blk] == 0x7FC0).all(), (t, q)
        if integer:
            assert np.array_equal(full, formats.encode_bf16_rne(oar.gemm_ar(a_list, b_list).astype(np.float32)))
        sig = run.signals.cpu().numpy()
        assert not sig[:2 * world].any()
        done = sig[2 * world + world * run.ntiles:2 * world + world * run.ntiles + world]
        assert [done[s] for s in range(world) if s != d] == [run.epoch] * (world - 1)


def test_flags_preset_waits_for_own_tiles_only(B):
    """DITRON_FLAGS_PRESET: the peers' partials are complete in memory; only this rank's tile flags are
    raised and waited for."""
    world, m_r, n, k, d = 4, 100, 264, 72, 3
    cfg = synth.CONFIGS[3].scaled(world=world, m_per_rank=m_r, n=n, k=k)
    a_list, b_list = synth.gemm_rs_inputs(cfg, integer=True)
    parts = [to_dev(oar.partial_bits(a, b)) for a, b in zip(a_list, b_list)]
    run = GemmArRun(B, world, cfg.m, n, k)
    peers = [None if s == d else parts[s] for s in range(world)]
    st = run(to_dev(a_list[d]), to_dev(nk(b_list[d])), peers, d, flags=B.FLAGS_PRESET)
    _ok(B, st, run)
    assert np.array_equal(bits(run.out), formats.encode_bf16_rne(oar.gemm_ar(a_list, b_list).astype(np.float32)))
    flags = run.signals.cpu().numpy()[2 * world:2 * world + world * run.ntiles].reshape(world, run.ntiles)
    for s in range(world):
        assert flags[s].tolist() == [run.epoch if s == d else 0] * run.ntiles
