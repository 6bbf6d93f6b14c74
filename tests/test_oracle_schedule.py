"""Pins for the integer schedule oracles: bijections, the paper's worked tiling example,
the arrival-order property the swizzle exists for, the agreement of the multi-node
listings with the single-node rotation when there is one node, and counter conservation."""
import os
import itertools
import pytest

from oracle import schedule as S
from oracle import ag_gemm as oag, gemm_rs as ors

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    for line in open(os.path.join(GOLD, path)):
        if not line.startswith("#") and line.strip():
            yield line.split()


@pytest.mark.parametrize("npm,npn,g", [(32, 14, 8), (7, 3, 4), (1, 1, 8), (5, 9, 1), (33, 2, 8)])
def test_grouped_order_is_bijection_and_row_fastest(npm, npn, g):
    seen = [S.grouped_order(p, npm, npn, g) for p in range(npm * npn)]
    assert sorted(seen) == sorted(itertools.product(range(npm), range(npn)))
    # inside a full group the tile row advances first
    if npm >= g and g > 1:
        assert seen[0] == (0, 0) and seen[1] == (1, 0) and seen[g] == (0, 1)


def test_grouped_order_group_1_is_row_major():
    assert [S.grouped_order(p, 3, 4, 1) for p in range(12)] == list(itertools.product(range(3), range(4)))


@pytest.mark.parametrize("ntiles", [1, 7, 8, 255, 256, 257, 448, 1024, 1000])
def test_xcd_remap_bijection_and_contiguity(ntiles):
    pids = [S.xcd_remap(w, ntiles) for w in range(ntiles)]
    assert sorted(pids) == list(range(ntiles))
    for base in range(0, ntiles, 256):
        size = min(256, ntiles - base)
        # a block maps onto itself: chip-wide waves keep the schedule's order
        assert sorted(pids[base:base + size]) == list(range(base, base + size))
        for x in range(8):
            mine = [pids[w] for w in range(base, base + size) if w % 8 == x]
            assert mine == list(range(mine[0], mine[0] + len(mine))) if mine else True


def test_ag_schedule_visits_shards_in_arrival_order():
    world, m_r, bm, n, bn = 8, 1024, 256, 3584, 256
    m = world * m_r
    for rank in range(world):
        order = []
        tiles = set()
        for pid in range(S.cdiv(m, bm) * S.cdiv(n, bn)):
            pm, pn, rb, re = S.ag_tile(pid, m, n, bm, bn, 1, rank, world)   # group 1: row-major time order
            tiles.add((pm, pn))
            assert rb == re == (pm * bm) // m_r
            if not order or order[-1] != rb:
                order.append(rb)
        assert order == oag.arrival_order(rank, world)
        assert len(tiles) == S.cdiv(m, bm) * S.cdiv(n, bn)
        # first tile is on the first row of the rank's own shard
        assert S.ag_tile(0, m, n, bm, bn, 8, rank, world)[0] * bm == rank * m_r


def test_ag_wait_set_straddling_tiles():
    # decode shape: 8 shards of 16 rows, one 128-row tile waits for all of them
    assert S.ag_tile(0, 128, 8192, 128, 128, 8, 3, 8)[2:] == (0, 7)
    # ragged: m_r = 100, bm = 64: tile row 1 covers rows 64..127 -> shards 0 and 1
    pm, pn, rb, re = S.ag_tile(0, 400, 64, 64, 64, 1, 0, 4)
    assert (pm, rb, re) == (0, 0, 0)
    got = {S.ag_tile(p, 400, 64, 64, 64, 1, 0, 4)[0]: S.ag_tile(p, 400, 64, 64, 64, 1, 0, 4)[2:] for p in range(7)}
    assert got[1] == (0, 1) and got[6] == (3, 3) and got[4] == (2, 3)
    # rank 1 starts at the first tile row lying entirely at or after row 100 -> ceil(100/64) = 2
    assert S.ag_tile(0, 400, 64, 64, 64, 1, 1, 4)[0] == 2


def test_rs_perfect_tiling_example_from_paper():
    (world, m_r, bm, per_rank), = [tuple(map(int, r)) for r in _rows("rs_perfect_tiling_example.txt")]
    m, n, bn = world * m_r, 256, 256
    npm = S.cdiv(m, bm)
    assert npm == world * per_rank
    for rank in range(world):
        rows = [S.rs_tile(p, m, n, bm, bn, 1, rank, world) for p in range(npm)]
        # tile row t belongs to exactly one rank: chunks [4i, 4i+4) go to rank i
        for pm, pn, s0, s1 in rows:
            assert s0 == s1 == pm // per_rank
        assert sorted(r[0] for r in rows) == list(range(npm))
        # scatter mode: begin with the next rank's chunk, own chunk last
        assert rows[0][0] == (per_rank * (rank + 1)) % npm
        assert [r[2] for r in rows[-per_rank:]] == [rank] * per_rank
    # with swizzling no two ranks work for the same destination at the same time
    for step in range(npm):
        dests = [S.rs_tile(step, m, n, bm, bn, 1, rank, world)[2] for rank in range(world)]
        assert len(set(dests)) == world
    # ... whereas the unswizzled order has every rank on destination 0 at step 0
    assert len({(S.grouped_order(0, npm, 1, 1)[0] * bm) // m_r for _ in range(world)}) == 1


def test_rs_completion_order_matches_arrival_order():
    world, m_r, bm = 8, 1024, 256
    m = world * m_r
    for d in range(world):
        # step at which rank s finishes destination d's segment
        finish = {}
        for s in range(world):
            for p in range(S.cdiv(m, bm)):
                pm, _, s0, _ = S.rs_tile(p, m, 256, bm, 256, 1, s, world)
                if s0 == d:
                    finish[s] = p
        assert sorted(range(world), key=lambda s: finish[s]) == ors.arrival_order(d, world)


@pytest.mark.parametrize("world,m_r,bm,bn,n", [(8, 1024, 256, 256, 8192), (4, 100, 64, 64, 200), (8, 997, 256, 256, 512)])
def test_rs_counter_conservation(world, m_r, bm, bn, n):
    m = world * m_r
    npm, npn = S.cdiv(m, bm), S.cdiv(n, bn)
    hits = [0] * world
    for pid in range(npm * npn):
        pm, pn, s0, s1 = S.rs_tile(pid, m, n, bm, bn, 8, 2 % world, world)
        assert 0 <= s0 <= s1 < world
        for seg in range(s0, s1 + 1):
            hits[seg] += 1
    for seg in range(world):
        assert hits[seg] == S.rs_segment_target(seg, m, n, bm, bn, world)
    if m_r % bm == 0:
        assert sum(hits) == npm * npn


@pytest.mark.parametrize("world,m_r,bm", [(8, 1024, 256), (8, 997, 256), (4, 100, 64), (2, 128, 256), (8, 16, 128)])
def test_multinode_listing_with_one_node_equals_single_node_rotation(world, m_r, bm):
    m = world * m_r
    npm = S.cdiv(m, bm)
    for rank in range(world):
        for t in range(npm):
            assert S.ag_swizzle_multinode(t, m, rank, world, 1, bm) == (t + S.cdiv(rank * m_r, bm)) % npm
            assert S.rs_swizzle_multinode(t, m, rank, world, 1, bm) == (t + ((rank + 1) * m_r) // bm) % npm


def test_multinode_swizzles_nonperfect_example_are_bijections():
    for world, nnodes, m_r, bm in [tuple(map(int, r)) for r in _rows("nonperfect_tiling_example.txt")]:
        m = world * m_r
        npm = S.cdiv(m, bm)
        for rank in range(world):
            ag = [S.ag_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]
            rs = [S.rs_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]
            assert sorted(ag) == list(range(npm)), (world, rank)
            assert sorted(rs) == list(range(npm)), (world, rank)


def test_multinode_perfect_tiling_properties():
    world, nnodes, m_r, bm = 16, 2, 1024, 256
    m = world * m_r
    npm, per_rank, local = S.cdiv(m, bm), m_r // bm, world // nnodes
    for rank in range(world):
        node = rank // local
        ag = [S.ag_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]
        rs = [S.rs_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]
        # gather mode: own rows first, and the whole own node before any other node
        assert ag[0] == rank * per_rank
        assert {(t * bm) // (m // nnodes) for t in ag[:npm // nnodes]} == {node}
        # scatter mode: next node first, own node (and inside it own rank) last
        assert {(t * bm) // (m // nnodes) for t in rs[:npm // nnodes]} == {(node + 1) % nnodes}
        assert [(t * bm) // m_r for t in rs[-per_rank:]] == [rank] * per_rank
    for step in range(npm):
        dests = {(S.rs_swizzle_multinode(step, m, r, world, nnodes, bm) * bm) // m_r for r in range(world)}
        assert len(dests) == world


# ---------------------------------------------------------------- ownership of shared tile rows
def _golden_orders():
    for ln in open(os.path.join(GOLD, "multinode_order_three_nodes.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        head, tail = ln.split(":")
        mode, world, nnodes, m_r, bm, rank = head.split()
        yield (mode,) + tuple(map(int, (world, nnodes, m_r, bm, rank))) + (list(map(int, tail.split())),)


def _oracle_order(mode, world, nnodes, m_r, bm, rank):
    f = S.ag_swizzle_multinode if mode == "gather" else S.rs_swizzle_multinode
    m = world * m_r
    return [f(t, m, rank, world, nnodes, bm) for t in range(S.cdiv(m, bm))]


def test_multinode_orders_worked_by_hand_three_nodes():
    """Seven orders worked by hand from the two listings for a shape whose node boundaries cut
    tile rows 3 and 6 (3 nodes, so the first, a middle and the last visit position all occur)."""
    cases = list(_golden_orders())
    assert len(cases) == 7
    for mode, world, nnodes, m_r, bm, rank, want in cases:
        assert _oracle_order(mode, world, nnodes, m_r, bm, rank) == want, (mode, rank)


def _order_from_ownership_rule(mode, world, nnodes, m_r, bm, rank):
    """The same order stated through sets instead of per-lane arithmetic.  Every tile row is owned
    by one node: a row holding rows of two nodes goes to the one visited LATER in gather order
    (both nodes' data must have arrived) and to the one visited EARLIER in scatter order (it is
    computed as early as possible for both).  Nodes are visited starting at the own node (gather)
    or the next one (scatter); inside a node's block of rows the visit starts at the tile row of
    the own local rank's first row (gather: first tile row starting at or after it; scatter: the
    tile row holding the next local rank's first row), never before the block's first row, and
    wraps around the block."""
    m = world * m_r
    m_node, local_world = m // nnodes, world // nnodes
    node_id, local_rank = rank // local_world, rank % local_world
    first = node_id if mode == "gather" else node_id + 1
    visit = [(first + p) % nnodes for p in range(nnodes)]
    when = {node: p for p, node in enumerate(visit)}
    owned = {node: [] for node in visit}
    for t in range(S.cdiv(m, bm)):
        touching = sorted({row // m_node for row in range(t * bm, min((t + 1) * bm, m))})
        assert len(touching) <= 2
        pick = max if mode == "gather" else min
        owned[pick(touching, key=lambda nd: when[nd])].append(t)
    order = []
    for node in visit:
        rows = owned[node]
        if mode == "gather":
            start = S.cdiv(m_node * node + m_r * local_rank, bm)
        else:
            start = (m_node * node + m_r * (local_rank + 1)) // bm
        shift = max(0, start - rows[0]) % len(rows)
        order += rows[shift:] + rows[:shift]
    return order


@pytest.mark.parametrize("world,nnodes,m_r,bm", [(8, 1, 997, 256), (16, 2, 997, 256), (32, 4, 997, 256), (6, 3, 100, 64),
                                                (12, 3, 77, 32), (16, 4, 1000, 128), (8, 2, 505, 256), (20, 5, 333, 128)])
def test_multinode_orders_follow_the_ownership_rule(world, nnodes, m_r, bm):
    for rank in range(world):
        for mode in ("gather", "scatter"):
            assert _oracle_order(mode, world, nnodes, m_r, bm, rank) == \
                _order_from_ownership_rule(mode, world, nnodes, m_r, bm, rank), (mode, rank)


def test_swapped_ownership_is_caught(monkeypatch):
    """Planting the mistake the pins exist for: with the gather and scatter ownership conditions
    exchanged the orders are still permutations, but neither the hand-worked table nor the
    ownership rule agrees any more."""
    real = S._node_blocks
    monkeypatch.setattr(S, "_node_blocks", lambda m, nn, bm, ns, mode: real(m, nn, bm, ns, "rs" if mode == "ag" else "ag"))
    wrong = 0
    for mode, world, nnodes, m_r, bm, rank, want in _golden_orders():
        got = _oracle_order(mode, world, nnodes, m_r, bm, rank)
        assert sorted(got) == list(range(len(want)))
        wrong += got != want
    assert wrong >= 5
    assert _oracle_order("gather", 16, 2, 997, 256, 3) != _order_from_ownership_rule("gather", 16, 2, 997, 256, 3)
