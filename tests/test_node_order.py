"""The multi-node tile-row order of the library (host evaluation of the function the kernels use)
against the oracle's restatement of the paper's two swizzle listings.  No GPU needed."""
import os

import pytest

from oracle import schedule as S


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    return binding


def _rows(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    return [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]


CASES = [(8, 1, 1024, 256), (16, 2, 1024, 256), (8, 2, 997, 256), (16, 2, 997, 256), (32, 4, 997, 256),
         (8, 4, 100, 64), (16, 4, 1000, 128), (8, 2, 16, 128), (32, 8, 300, 256), (12, 3, 77, 32)]


@pytest.mark.parametrize("world,nnodes,m_r,bm", CASES)
def test_library_order_equals_oracle(B, world, nnodes, m_r, bm):
    m = world * m_r
    npm = S.cdiv(m, bm)
    for rank in range(world):
        st, got = B.tile_row_order(0, m, bm, world, nnodes, rank)
        assert st == B.OK
        assert got == [S.ag_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]
        st, got = B.tile_row_order(1, m, bm, world, nnodes, rank)
        assert st == B.OK
        assert got == [S.rs_swizzle_multinode(t, m, rank, world, nnodes, bm) for t in range(npm)]


def test_paper_nonperfect_example_is_visited_once(B):
    # the shapes of the paper's non-perfect tiling example (997 rows per rank; 8, 16, 32 GPUs)
    for world, nnodes, m_r, bm in [tuple(map(int, r)) for r in _rows("nonperfect_tiling_example.txt")]:
        m = world * m_r
        for rank in range(world):
            for op in (0, 1):
                st, got = B.tile_row_order(op, m, bm, world, nnodes, rank)
                assert st == B.OK and sorted(got) == list(range(S.cdiv(m, bm)))


def test_one_node_is_the_plain_rotation(B):
    world, m_r, bm = 8, 505, 256
    m = world * m_r
    npm = S.cdiv(m, bm)
    for rank in range(world):
        assert B.tile_row_order(0, m, bm, world, 1, rank)[1] == [(t + S.cdiv(rank * m_r, bm)) % npm for t in range(npm)]
        assert B.tile_row_order(1, m, bm, world, 1, rank)[1] == [(t + ((rank + 1) * m_r) // bm) % npm for t in range(npm)]


def test_argument_checks(B):
    assert B.tile_row_order(2, 1024, 256, 8, 2, 0)[0] == B.ERR_INVALID_ARG       # unknown order
    assert B.tile_row_order(0, 1024, 256, 8, 3, 0)[0] == B.ERR_INVALID_ARG       # world not a multiple of nnodes
    assert B.tile_row_order(0, 1000, 256, 8, 2, 8)[0] == B.ERR_INVALID_ARG       # rank out of range
    assert B.tile_row_order(0, 1001, 256, 8, 2, 0)[0] == B.ERR_INVALID_ARG       # rows not a multiple of world
