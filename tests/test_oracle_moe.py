"""Pins for the MoE routing / schedule / grouped-GEMM oracles: conservation, agreement
with numpy's stable argsort and bincount, brute force on tiny inputs, degenerate routings,
and an independent derivation of each tile's source-rank span."""
import numpy as np
import pytest

import synth
from oracle import moe, formats
from oracle import ag_gemm as oag
from oracle.schedule import cdiv


def _ids(tokens, experts, top_k, seed=0):
    return synth.routing_topk(np.random.default_rng(seed), tokens, experts, top_k)


def test_routing_draw_is_distinct_and_uniformish():
    ids = _ids(4096, 64, 2)
    assert ids.dtype == np.int32 and ids.shape == (4096, 2)
    assert (ids[:, 0] != ids[:, 1]).all() and ids.min() >= 0 and ids.max() < 64
    c = np.bincount(ids.reshape(-1), minlength=64)
    assert c.min() > 60 and c.max() < 200     # mean 128


@pytest.mark.parametrize("world,t_r,experts,top_k,e0,el", [(8, 64, 64, 2, 8, 8), (4, 16, 8, 2, 0, 8), (2, 8, 6, 3, 2, 3)])
def test_route_vs_numpy_library(world, t_r, experts, top_k, e0, el):
    ids = _ids(world * t_r, experts, top_k, seed=world)
    count, offsets, gather = moe.route(ids, world, experts, e0, el)
    assert count.sum() == world * t_r * top_k
    flat = ids.reshape(-1)
    shard_of = np.arange(flat.size) // (t_r * top_k)
    for s in range(world):
        assert np.array_equal(count[s], np.bincount(flat[shard_of == s], minlength=experts))
    order = np.argsort(flat, kind="stable")
    local = order[(flat[order] >= e0) & (flat[order] < e0 + el)]
    assert np.array_equal(gather, local)
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=experts)[e0:e0 + el])]))
    for j in range(el):
        seg = gather[offsets[j]:offsets[j + 1]]
        assert (flat[seg] == e0 + j).all() and (np.diff(seg) > 0).all()


def test_route_degenerate_cases():
    # everything to one expert
    ids = np.full((12, 1), 3, dtype=np.int32)
    count, offsets, gather = moe.route(ids, 4, 5, 2, 3)
    assert list(offsets) == [0, 0, 12, 12] and list(gather) == list(range(12))
    assert count[:, 3].tolist() == [3, 3, 3, 3]
    # no token for the local experts
    count, offsets, gather = moe.route(ids, 4, 5, 0, 2)
    assert list(offsets) == [0, 0, 0] and gather.size == 0
    # tiny brute force
    ids = np.array([[1, 0], [2, 1], [0, 2], [1, 2]], dtype=np.int32)
    count, offsets, gather = moe.route(ids, 2, 3, 1, 2)
    assert list(offsets) == [0, 3, 6]
    assert list(gather) == [0, 3, 6, 2, 5, 7]
    assert count.tolist() == [[1, 2, 1], [1, 1, 2]]


@pytest.mark.parametrize("rank", [0, 3, 7])
@pytest.mark.parametrize("bm", [16, 64, 128])
def test_tile_schedule_invariants(rank, bm):
    world, t_r, experts, top_k, el = 8, 128, 16, 2, 4
    e0 = (rank * el) % experts
    ids = _ids(world * t_r, experts, top_k, seed=rank)
    count, offsets, gather = moe.route(ids, world, experts, e0, el)
    sch = moe.tile_schedule(count, e0, el, bm, rank, world)
    n_e = [int(offsets[j + 1] - offsets[j]) for j in range(el)]
    assert sch["ntiles"] == sum(cdiv(n, bm) for n in n_e)
    assert sorted(sch["tiled_m"]) == list(range(sch["ntiles"]))
    first_tile = np.concatenate([[0], np.cumsum([cdiv(n, bm) for n in n_e])])
    pos = 0
    for j in range(el):
        stages = []
        for _ in range(cdiv(n_e[j], bm)):
            assert sch["expert_id"][pos] == j
            tau = sch["tiled_m"][pos]
            assert first_tile[j] <= tau < first_tile[j + 1]
            # independent derivation: source ranks of the tile's first / last gathered row
            q0 = (tau - first_tile[j]) * bm
            q1 = min(q0 + bm, n_e[j])
            src = (gather[offsets[j] + q0: offsets[j] + q1] // top_k) // t_r
            assert sch["segment_start"][pos] == src[0] == src.min()
            assert sch["segment_end"][pos] == src[-1] == src.max()
            # the stage is the delivery position, in the producer's order, of the last shard needed
            ring = oag.arrival_order(rank, world)
            assert sch["stage"][pos] == max(ring.index(int(s)) for s in src)
            stages.append((sch["stage"][pos], tau))
            pos += 1
        assert stages == sorted(stages)      # ascending stage, ties by original index
    assert pos == sch["ntiles"]


def test_tile_schedule_tiny_by_hand():
    # 2 ranks, 1 local expert (id 0): rank0 sends 3 rows, rank1 sends 2 rows; tiles of 2 rows
    count = np.array([[3], [2]])
    sch = moe.tile_schedule(count, 0, 1, 2, rank=1, world=2)
    # tiles: rows [0,2) from rank 0 ; [2,4) ranks 0..1 ; [4,5) rank 1.  For rank 1 the ring
    # order is 1, 0: the tile needing only rank 1 has stage 0, the others stage 1.
    assert sch["ntiles"] == 3
    assert sch["tiled_m"] == [2, 0, 1]
    assert sch["segment_start"] == [1, 0, 0] and sch["segment_end"] == [1, 0, 1]
    assert sch["stage"] == [0, 1, 1]
    # empty expert in front
    count = np.array([[0, 1], [0, 1]])
    sch = moe.tile_schedule(count, 0, 2, 4, rank=0, world=2)
    assert sch["ntiles"] == 1 and sch["expert_id"] == [1] and sch["segment_start"] == [0] and sch["segment_end"] == [1]


def test_tile_stage_follows_the_producers_delivery_order_by_hand():
    """The all-gather producer delivers to rank r in the order r, r+1, ... (mod W).  With 3 ranks and
    rank 1 the order is 1, 2, 0, which a ring walked the other way (1, 0, 2) does not share."""
    assert oag.arrival_order(1, 3) == [1, 2, 0]
    # one local expert, 2 rows from every rank, tiles of 2 rows: tile t holds exactly rank t's rows
    count = np.array([[2], [2], [2]])
    sch = moe.tile_schedule(count, 0, 1, 2, rank=1, world=3)
    # rank 1's own rows are there first (stage 0), then rank 2's (stage 1), rank 0's last (stage 2)
    assert sch["tiled_m"] == [1, 2, 0]
    assert sch["stage"] == [0, 1, 2]
    assert sch["segment_start"] == [1, 2, 0] and sch["segment_end"] == [1, 2, 0]
    # 4 ranks, rank 2 (delivery order 2, 3, 0, 1); rows per rank 3, 1, 2, 2; tiles of 3 rows:
    #   tile 0 = rows 0..2  (rank 0)          -> waits for delivery position 2
    #   tile 1 = rows 3..5  (ranks 1, 2, 2)   -> ranks 1..2, the later of positions 3 and 0 = 3
    #   tile 2 = rows 6..7  (ranks 3, 3)      -> position 1
    assert oag.arrival_order(2, 4) == [2, 3, 0, 1]
    count = np.array([[3], [1], [2], [2]])
    sch = moe.tile_schedule(count, 0, 1, 3, rank=2, world=4)
    assert sch["tiled_m"] == [2, 0, 1]
    assert sch["stage"] == [1, 2, 3]
    assert sch["segment_start"] == [3, 0, 1] and sch["segment_end"] == [3, 0, 2]


def test_reversed_ring_is_caught(monkeypatch):
    """Planting the mistake: with the ring walked backwards the stage is still a permutation of
    0..W-1 over the shards, every invariant test still holds, but the hand-worked orders differ."""
    for rank, world in [(1, 3), (2, 4), (5, 8)]:
        assert [moe.stage_of_shard(s, rank, world) for s in oag.arrival_order(rank, world)] == list(range(world))
    monkeypatch.setattr(moe, "stage_of_shard", lambda s, rank, world: (rank - s) % world)
    sch = moe.tile_schedule(np.array([[2], [2], [2]]), 0, 1, 2, rank=1, world=3)
    assert sch["tiled_m"] == [1, 0, 2] != [1, 2, 0]
    with pytest.raises(AssertionError):
        test_tile_stage_follows_the_producers_delivery_order_by_hand()


def test_grouped_gemm_brute_force_tiny():
    cfg = synth.CONFIGS[4].scaled(world=2, tokens_per_rank=3, k=4, n=3, num_experts=4, top_k=2,
                                  num_local_experts=2, rank=1)
    xs, ids, w = synth.moe_inputs(cfg)
    e0 = cfg.rank * cfg.num_local_experts
    y = moe.grouped_gemm(xs, ids, w, cfg.world, cfg.num_experts, e0)
    x = np.concatenate([formats.decode_bf16(s) for s in xs])
    wd = formats.decode_bf16(w)
    rows = []
    for e in range(e0, e0 + 2):
        for t in range(6):
            for j in range(2):
                if ids[t, j] == e:
                    rows.append([sum(x[t, h] * wd[e - e0, h, c] for h in range(4)) for c in range(3)])
    assert y.shape == (len(rows), 3)
    assert np.allclose(y, np.array(rows).reshape(len(rows), 3), rtol=1e-13, atol=1e-13)
    xg = moe.gather_rows(xs, moe.route(ids, 2, 4, e0, 2)[2], 2)
    assert xg.dtype == np.uint16 and xg.shape == (len(rows), 4)
