"""CPU-side checks of the C ABI: the library loads, exports every function the header
declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ditron.h")


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    return binding


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ditron_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = _declared_functions()
    assert {"ditron_ag_gemm", "ditron_gemm_rs", "ditron_moe_ag_grouped_gemm", "ditron_reduce_slots",
            "ditron_publish_chunks", "ditron_tile_config", "ditron_signal_words", "ditron_gemm_ar"} <= set(names)
    for n in names:
        assert hasattr(B.lib, n), n


def test_sizes_and_strings(B):
    assert B.signal_words(8, 1) == 48 and B.signal_words(8, 4) == 96 and B.signal_words(0, 1) == 0
    # the gathered operand: world * rows * k elements of the operand type
    assert B.ag_gemm_workspace_bytes(1024, 3584, 8192, 8) == 8 * 1024 * 8192 * 2
    # decode shape: the gathered fp8 operand, then 64 tiles x 4 splits of 128 x 128 partials of 8 bytes (value, epoch)
    assert B.ag_gemm_workspace_bytes(16, 8192, 8192, 8, B.FP8_E4M3) == 128 * 8192 + 64 * 4 * 128 * 128 * 8
    assert B.ag_gemm_workspace_bytes(16, 8192, 8192, 8, B.FP8_E4M3, tuning=B.tuning(decode_variant=1)) == 128 * 8192
    assert B.ag_gemm_workspace_bytes(0, 8, 8192, 8) == 0 and B.ag_gemm_workspace_bytes(16, 8, 8192, 8, 5) == 0
    assert B.moe_workspace_bytes(1024, 4096, 8) == 8 * 1024 * 4096 * 2 + B.MOE_ROUTE_SCRATCH_BYTES and B.moe_workspace_bytes(1024, 0, 8) == 0
    assert B.status_string(B.OK) == "ok" and "time" in B.status_string(B.ERR_TIMEOUT)
    assert B.moe_max_tiles(4096, 8) == 4096 // 128 + 8


def test_tile_config(B):
    st, tc = B.tile_config(0, 8192, 3584, 8192)
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"]) == (256, 224, 512)   # two whole rounds instead of 1.75
    st, tc = B.tile_config(0, 256, 256, 256)           # few tiles, B stored [n, k]: the decode kernel's 128 x 128 tile
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"], tc["splits"]) == (128, 128, 4, 1)
    st, tc = B.tile_config(0, 256, 256, 256, tuning=B.tuning(decode_variant=1))
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"], tc["splits"]) == (128, 32, 16, 1)
    st, tc = B.tile_config(4, 256, 256, 256)           # B stored [k, n]: the tile engine
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"]) == (128, 128, 4)
    st, tc = B.tile_config(0, 2048, 2048, 256)
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"]) == (128, 128, 256)
    st, tc = B.tile_config(0, 128, 8192, 8192, B.FP8_E4M3)     # the decode shape: 64 tiles, the contraction split in 4
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"], tc["splits"]) == (128, 128, 64, 4)
    st, tc = B.tile_config(0, 128, 8192, 8192, B.FP8_E4M3, B.tuning(decode_variant=3))
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"], tc["splits"]) == (128, 64, 128, 2)
    st, tc = B.tile_config(0, 128, 8192, 8192, B.FP8_E4M3, B.tuning(decode_variant=4))     # one tile per shard and column block
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"], tc["splits"]) == (16, 128, 512, 1)
    # the column count of the 256-row tile: 224 or 192 where that fills the last round of 256 units better (AllGather-GEMM with B
    # stored [n, k] only), 256 otherwise
    assert B.tile_config(0, 8192, 8192, 3584)[1]["block_n"] == 256      # four whole rounds of 256-column tiles
    assert B.tile_config(0, 8192, 3696, 8192)[1]["block_n"] == 256      # 480 tiles of 256 columns against 544 of 224
    assert B.tile_config(0, 8192, 6656, 16384)[1]["block_n"] == 224     # 3.75 rounds of 224-column tiles against 3.25 of 256
    assert B.tile_config(0, 8192, 1792, 4096)[1]["block_n"] == 224      # 8 x 224 columns: one whole round
    assert B.tile_config(0, 8192, 1376, 4096)[1]["block_n"] == 192      # 8 x 192 columns: one whole round against 0.75 (256) or 0.875 (224)
    assert B.tile_config(4, 8192, 3584, 8192)[1]["block_n"] == 256      # B stored [k, n]
    assert B.tile_config(1, 8192, 3584, 8192)[1]["block_n"] == 256 and B.tile_config(3, 8192, 3584, 8192)[1]["block_n"] == 256
    assert B.tile_config(7, 1, 1, 1)[0] == B.ERR_INVALID_ARG


def test_operand_staging_choice(B):
    """256 x 256 tiles of [n, k] operands take the direct-to-LDS staging, whatever the contraction length."""
    assert B.tile_config(0, 8192, 3584, 8192)[1]["direct_staging"] == 1      # cfg 2
    assert B.tile_config(1, 8192, 8192, 3584)[1]["direct_staging"] == 1      # cfg 3
    assert B.tile_config(3, 8192, 8192, 3584)[1]["direct_staging"] == 1
    assert B.tile_config(0, 8192, 6656, 16384)[1]["direct_staging"] == 1     # long contraction
    assert B.tile_config(0, 8192, 6656, 12288)[1]["direct_staging"] == 1 and B.tile_config(0, 8192, 6656, 12360)[1]["direct_staging"] == 1
    assert B.tile_config(1, 8192, 8192, 3696)[1]["direct_staging"] == 1      # ragged last K tile
    assert B.tile_config(4, 8192, 3584, 8192)[1]["direct_staging"] == 0      # B stored [k, n]
    assert B.tile_config(0, 2048, 2048, 256)[1]["direct_staging"] == 0       # 128 x 128 tiles
    assert B.tile_config(0, 128, 8192, 8192, B.FP8_E4M3)[1]["direct_staging"] == 0


def test_moe_tile_choice(B):
    """Host rule for the grouped GEMM's tile: 256 rows when an expert expects 1024 rows or more, or when
    rounds x (rows + columns) of the 256-row tiling is below that of the 128-row tiling by more than 1.3; for
    128-row tiles the narrowest column block that keeps one tile per compute unit (256 of them) with a
    row tile to spare, else the block that pads the intermediate size least, the wider on a tie."""
    # cfg 4: 8192 tokens, top-2 of 64 experts, 8 local -> 2048 rows, 16 + 4 row tiles; 21 x 12 blocks of 128 fit
    assert B.moe_tile_choice(8192, 2, 64, 8, 1536) == (B.OK, 128, 128)
    # one row tile more (22 x 12 = 264 > 256): 192 columns (22 x 8)
    assert B.moe_tile_choice(8192 + 128 * 4, 2, 64, 8, 1536) == (B.OK, 128, 192)
    # many tiles (two rounds with either row tile), 176 columns: 192 pads least; 256 columns: 128 and 256 tie,
    # the wider wins
    assert B.moe_tile_choice(14592, 4, 60, 60, 176) == (B.OK, 128, 192)
    assert B.moe_tile_choice(14400, 4, 64, 64, 256) == (B.OK, 128, 256)
    # the paper's two many-expert shapes: 286 / 416 tiles of 128 rows need two rounds, 256-row tiles one
    assert B.moe_tile_choice(8192, 4, 60, 60, 176) == (B.OK, 256, 256)
    assert B.moe_tile_choice(8192, 6, 64, 64, 256) == (B.OK, 256, 256)
    # 2048 rows per expert: the 256-row tile, 256 columns unless the intermediate size is at most 128
    assert B.moe_tile_choice(8192, 2, 8, 8, 512) == (B.OK, 256, 256)
    assert B.moe_tile_choice(8192, 2, 8, 8, 128) == (B.OK, 256, 128)
    assert B.moe_tile_choice(0, 2, 8, 8, 128)[0] == B.ERR_INVALID_ARG
    assert B.moe_tile_choice(8192, 2, 8, 9, 128)[0] == B.ERR_INVALID_ARG


def test_ag_gemm_argument_checks(B):
    null = None
    fake = 0x1000          # never dereferenced: the checks fail first
    args = dict(a_shards=[fake, fake], b=fake, b_layout=B.B_NK, c=fake, a_scales=null, b_scales=null,
                workspace=fake, signals=fake, status=fake, schedule_out=null, arrival_order=null,
                m_per_rank=128, n=256, k=256, world=2, rank=0, dtype=B.BF16, epoch=1,
                flags=B.EMULATE_PRODUCER, stream=ctypes.c_void_p(0))

    def call(**kw):
        a = dict(args)
        a.update(kw)
        s = a.pop("stream")
        return B.lib.ditron_ag_gemm(B._ptr_array(a["a_shards"]), B._ptr(a["b"]), a["b_layout"], B._ptr(a["c"]),
                                    None, None, B._ptr(a["workspace"]), B._ptr(a["signals"]), B._ptr(a["status"]),
                                    B._ptr(a["schedule_out"]), B._int_array(a["arrival_order"]), a["m_per_rank"],
                                    a["n"], a["k"], a["world"], a["rank"], a["dtype"], a["epoch"], a["flags"],
                                    B._tuning(a.get("tuning")), s)

    assert call(world=0) == B.ERR_INVALID_ARG
    assert call(world=B.MAX_WORLD + 1, a_shards=[fake] * 40) == B.ERR_INVALID_ARG
    assert call(rank=2) == B.ERR_INVALID_ARG
    assert call(k=0) == B.ERR_INVALID_ARG
    assert call(b=null) == B.ERR_INVALID_ARG
    assert call(c=0x1008) == B.ERR_INVALID_ARG                       # misaligned
    assert call(flags=0) == B.ERR_INVALID_ARG                        # no producer mode
    assert call(flags=B.EMULATE_PRODUCER | B.EXTERNAL_PRODUCER) == B.ERR_INVALID_ARG
    assert call(flags=B.EMULATE_PRODUCER | B.DUMP_SCHEDULE) == B.ERR_INVALID_ARG   # no schedule buffer
    assert call(arrival_order=[0, 0]) == B.ERR_INVALID_ARG           # not a permutation
    assert call(a_shards=[fake, None]) == B.ERR_INVALID_ARG
    assert call(dtype=9) == B.ERR_INVALID_ARG
    assert call(b_layout=7) == B.ERR_INVALID_ARG
    assert call(b_layout=B.B_KN, dtype=B.FP8_E4M3) == B.ERR_UNSUPPORTED   # the fp8 operator takes B as [n, k] only
    assert call(k=260) == B.ERR_UNSUPPORTED                          # contraction not a multiple of 8
    assert call(flags=B.FLAGS_PRESET | B.EXTERNAL_PRODUCER) == B.ERR_INVALID_ARG    # one producer mode at a time
    assert call(tuning=B.tuning(num_nodes=3)) == B.ERR_INVALID_ARG   # nodes must divide the ranks
    assert call(tuning=B.tuning(num_nodes=-1)) == B.ERR_INVALID_ARG
    bad = B.tuning()
    bad.reserved[2] = 1
    assert call(tuning=bad) == B.ERR_INVALID_ARG                     # reserved words must be zero


def test_gemm_rs_and_moe_argument_checks(B):
    fake = 0x1000
    z = ctypes.c_void_p(0)
    st = B.lib.ditron_gemm_rs(B._ptr(fake), B._ptr(fake), B.B_NK, B._ptr(fake), None, B._ptr(fake), B._ptr(fake),
                              B._ptr(fake), B._ptr(fake), None, None, 1000, 256, 64, 8, 0, 1, 1,
                              B.EMULATE_PRODUCER, None, z)
    assert st == B.ERR_INVALID_ARG          # m not divisible by world
    st = B.lib.ditron_gemm_rs(B._ptr(fake), B._ptr(fake), B.B_NK, B._ptr(fake), None, B._ptr(fake), B._ptr(fake),
                              B._ptr(fake), B._ptr(fake), None, None, 1024, 256, 64, 8, 0, 3, 1,
                              B.EMULATE_PRODUCER, None, z)
    assert st == B.ERR_INVALID_ARG          # chunks do not divide the rows per rank
    st = B.gemm_rs_fuse_scatter(fake, fake, B.B_NK, None, None, fake, fake, fake, None, None, 1024, 256, 64, 8, 0, 1, 1,
                                B.EMULATE_PRODUCER, stream=_S())
    assert st == B.ERR_INVALID_ARG          # no destination buffers
    st = B.gemm_rs_fuse_scatter(fake, fake, B.B_NK, [fake] * 7 + [None], [fake] * 8, fake, fake, fake, None, None, 1024,
                                256, 64, 8, 0, 1, 1, B.EMULATE_PRODUCER, stream=_S())
    assert st == B.ERR_INVALID_ARG          # a destination is missing
    st = B.lib.ditron_reduce_slots(None, B._ptr(fake), None, None, 8, 8, 2, 1, 1, None, z)
    assert st == B.ERR_INVALID_ARG
    st = B.moe_ag_grouped_gemm([fake] * 8, fake, fake, B.B_NK, fake, fake, fake, fake, fake, fake, fake, fake, None,
                               1024, 4096, 1536, 64, 2, 60, 8, 4096, 8, 0, 1, B.EMULATE_PRODUCER, stream=_S())
    assert st == B.ERR_INVALID_ARG          # local experts run past the expert count
    st = B.moe_ag_grouped_gemm([fake] * 8, fake, fake, B.B_NK, fake, fake, fake, fake, fake, fake, fake, fake, None,
                               1024, 4096, 1536, 512, 2, 0, 8, 4096, 8, 0, 1, B.EMULATE_PRODUCER, stream=_S())
    assert st == B.ERR_UNSUPPORTED          # more experts than the routing kernel holds
    st = B.publish_chunks([fake], [fake], [24], [0], fake, 1, stream=_S())
    assert st == B.ERR_INVALID_ARG          # size not a multiple of 16


def test_gemm_ar_argument_checks(B):
    fake, other = 0x1000, 0x2000
    args = dict(a=fake, b=fake, b_layout=B.B_NK, gemm_out=fake, peer_partials=[other] * 4, out=other + 0x1000,
                signals=fake, status=fake, schedule_out=None, m=256, n=256, k_local=64, world=4, rank=0, epoch=1,
                flags=B.EMULATE_PRODUCER)

    def call(**kw):
        a = dict(args)
        a.update(kw)
        return B.gemm_ar(stream=_S(), **a)

    assert call(world=0) == B.ERR_INVALID_ARG
    assert call(rank=4) == B.ERR_INVALID_ARG
    assert call(out=fake) == B.ERR_INVALID_ARG                        # output on top of the published partial
    assert call(peer_partials=None) == B.ERR_INVALID_ARG
    assert call(peer_partials=[other, None, other, other]) == B.ERR_INVALID_ARG
    assert call(flags=0) == B.ERR_INVALID_ARG
    assert call(flags=B.EMULATE_PRODUCER | B.DUMP_SCHEDULE) == B.ERR_INVALID_ARG   # no schedule buffer
    assert call(b_layout=5) == B.ERR_INVALID_ARG
    assert call(k_local=60) == B.ERR_UNSUPPORTED
    assert call(n=100) == B.ERR_UNSUPPORTED
    st, tc = B.tile_config(3, 8192, 8192, 3584)
    assert st == B.OK and (tc["block_m"], tc["block_n"], tc["ntiles"]) == (256, 256, 1024)


def test_schedule_dump_on_the_host(B):
    """The host evaluation of the schedule against the oracle's statement of the same arithmetic."""
    from oracle import schedule as S
    for op, m, n, k, world, rank, tile in [(0, 8192, 3584, 8192, 8, 3, S.ag_tile), (1, 8192, 8192, 3584, 8, 5, S.rs_tile),
                                           (0, 1616, 2056, 136, 8, 7, S.ag_tile), (1, 800, 264, 72, 4, 1, S.rs_tile)]:
        st, tc = B.tile_config(op, m, n, k)
        st, got = B.schedule_dump(op, m, n, k, world, rank)
        assert st == B.OK and len(got) == tc["ntiles"]
        want = [tile(S.xcd_remap(wg, tc["ntiles"], tc["num_xcd"], tc["per_xcd"]), m, n, tc["block_m"], tc["block_n"],
                     tc["group_m"], rank, world) for wg in range(tc["ntiles"])]
        assert got == want
    # GEMM + AllReduce: position -> tile, no rotation
    from oracle import gemm_ar as oar
    st, tc = B.tile_config(3, 1024, 2048, 64)
    st, got = B.schedule_dump(3, 1024, 2048, 64, 4, 2)
    assert st == B.OK and [g[:2] for g in got] == [oar.tile_at_position(t, 1024, 2048, tc["block_m"], tc["block_n"], tc["group_m"],
                                                                         tc["num_xcd"], tc["per_xcd"]) for t in range(tc["ntiles"])]
    # across nodes the order comes from the multi-node listings; a shape they do not cover is refused
    st, got = B.schedule_dump(0, 8 * 505, 3080, 64, 8, 5, tuning=B.tuning(num_nodes=4))
    st2, tc = B.tile_config(0, 8 * 505, 3080, 64)
    assert st == B.OK
    rows_in_order = []
    for g in got:
        if g[0] not in rows_in_order:
            rows_in_order.append(g[0])
    assert sorted(rows_in_order) == list(range(S.cdiv(8 * 505, tc["block_m"])))
    assert B.schedule_dump(0, 8 * 37, 128, 64, 8, 4, b_layout=B.B_KN, tuning=B.tuning(num_nodes=4))[0] == B.ERR_UNSUPPORTED
    # capacity too small: the count is still reported
    import ctypes as C
    cnt = C.c_int(0)
    out = (C.c_int32 * 4)()
    assert B.lib.ditron_schedule_dump(0, 8192, 3584, 8192, 8, 0, B.BF16, B.B_NK, None, out, 1, C.byref(cnt)) == B.ERR_WORKSPACE
    assert cnt.value == 512
    assert B.lib.ditron_schedule_dump(2, 8192, 3584, 8192, 8, 0, B.BF16, B.B_NK, None, out, 1, C.byref(cnt)) == B.ERR_INVALID_ARG
    assert B.lib.ditron_schedule_dump(0, 8192, 3584, 8192, 8, 8, B.BF16, B.B_NK, None, out, 1, C.byref(cnt)) == B.ERR_INVALID_ARG


class _S:
    cuda_stream = 0
