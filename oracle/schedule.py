"""Integer tile schedules (paper, Section "Mid-end Compute-Communication Swizzling",
Appendix "Swizzle", and the index arithmetic at the top of the AllGather-GEMM consumer and
GEMM-ReduceScatter producer kernels).

All quantities are non-negative Python ints; // is floor division.
"""


def cdiv(a, b):
    return -(-a // b)


def grouped_order(pid, num_pid_m, num_pid_n, group_m):
    """Linear tile id -> (pid_m, pid_n): tile rows are taken in groups of `group_m`; inside
    a group the row index runs fastest (AllGather-GEMM consumer kernel, first lines)."""
    in_group = group_m * num_pid_n
    group_id = pid // in_group
    first_m = group_id * group_m
    size_m = min(num_pid_m - first_m, group_m)
    pid_m = first_m + (pid % in_group) % size_m
    pid_n = (pid % in_group) // size_m
    return pid_m, pid_n


def xcd_remap(wg, ntiles, num_xcd=8, per_xcd=32):
    """Work-group index -> linear tile id.  Not from the paper: the GPU hands work-group w
    to chiplet w % num_xcd, and this bijection gives each chiplet a run of consecutive tile
    ids inside every block of num_xcd*per_xcd tiles, so that tiles sharing operand panels
    share an L2.  Blocks are taken in order, so the arrival-keyed order of the paper's
    schedule is kept at the granularity of one chip-wide wave of tiles.

    Built by construction: inside a block of size S, chiplet x owns the work-groups
    {w : w % num_xcd == x} in increasing w, and receives the next len(...) tile ids."""
    block = num_xcd * per_xcd
    base = (wg // block) * block
    size = min(block, ntiles - base)
    local = wg - base
    next_tile = base
    for x in range(num_xcd):
        members = [w for w in range(size) if w % num_xcd == x]
        if local % num_xcd == x:
            return next_tile + members.index(local)
        next_tile += len(members)
    raise AssertionError


def ag_tile(pid, m, n, block_m, block_n, group_m, rank, world):
    """AllGather-GEMM tile of linear id `pid`: returns (pid_m, pid_n, rank_beg, rank_end).
    The tile row is rotated so that rank r starts on the rows of its own shard, and the
    tile must wait for the shards rank_beg..rank_end that its rows touch."""
    npm, npn = cdiv(m, block_m), cdiv(n, block_n)
    pid_m, pid_n = grouped_order(pid, npm, npn, group_m)
    m_r = m // world
    pid_m = (pid_m + cdiv(m_r * rank, block_m)) % npm
    row0 = pid_m * block_m
    rank_beg = row0 // m_r
    rank_end = (min(row0 + block_m, m) - 1) // m_r
    return pid_m, pid_n, rank_beg, rank_end


def rs_tile(pid, m, n, block_m, block_n, group_m, rank, world):
    """GEMM-ReduceScatter tile of linear id `pid`: (pid_m, pid_n, segment_start,
    segment_end).  Rows are rotated so that the segment of rank r+1 is computed first and
    the rank's own segment last."""
    npm, npn = cdiv(m, block_m), cdiv(n, block_n)
    pid_m, pid_n = grouped_order(pid, npm, npn, group_m)
    m_r = m // world
    pid_m = (pid_m + ((rank + 1) * m_r) // block_m) % npm
    seg_start = (pid_m * block_m) // m_r
    seg_end = (min((pid_m + 1) * block_m, m) - 1) // m_r
    return pid_m, pid_n, seg_start, seg_end


def rs_segment_target(segment, m, n, block_m, block_n, world):
    """Number of tiles that must finish before segment `segment` is complete: every tile
    row that intersects the segment's rows, times the number of tile columns."""
    m_r = m // world
    first = (m_r * segment) // block_m
    last = (m_r * (segment + 1) - 1) // block_m
    return cdiv(n, block_n) * (last - first + 1)


# ---------------------------------------------------------------- multi-node swizzles
def _node_blocks(m, nnodes, block_m, node_start, mode):
    """Tile-row ranges [start, end] owned by each node, visited in the order
    node_start, node_start+1, ... (mod nnodes).  A tile row that straddles two nodes is
    given to exactly one of them, following the appendix listings: position 0 of the visit
    order behaves differently from the rest and the two modes differ in which side wins."""
    m_node = m // nnodes
    sizes, starts = [], []
    for pos in range(nnodes):
        node = (pos + node_start) % nnodes
        lo, hi = m_node * node, m_node * (node + 1)
        t_lo = lo // block_m
        t_hi = (hi - 1) // block_m
        prev_end = (lo - 1) // block_m if lo != 0 else -1
        next_start = hi // block_m
        if mode == "ag":
            if pos == 0 and lo != 0 and prev_end == t_lo:
                t_lo += 1
            if pos == 0 and hi != m and next_start == t_hi:
                t_hi -= 1
            if pos != nnodes - 1 and hi != m and next_start == t_hi:
                t_hi -= 1
        else:
            if pos != 0 and lo != 0 and prev_end == t_lo:
                t_lo += 1
            if pos == nnodes - 1 and hi != m and next_start == t_hi:
                t_hi -= 1
        starts.append(t_lo)
        sizes.append(t_hi - t_lo + 1)
    return starts, sizes


def _multinode_swizzle(tiled_m, m, rank, world, nnodes, block_m, mode):
    local_world = world // nnodes
    node_id = rank // local_world
    m_r = m // world
    m_node = m // nnodes
    node_start = (node_id + (0 if mode == "ag" else 1)) % nnodes
    _, sizes_by_pos = _node_blocks(m, nnodes, block_m, node_start, mode)
    # which visit position does tiled_m fall in (positions are laid out one after another)
    acc = 0
    pos = None
    for p in range(nnodes):
        if tiled_m < acc + sizes_by_pos[p]:
            pos = p
            break
        acc += sizes_by_pos[p]
    assert pos is not None, "tiled_m beyond the swizzled range"
    offset_in_order = acc
    tile_size = sizes_by_pos[pos]
    nid = (pos + node_start) % nnodes
    # sizes indexed by node id, and their exclusive prefix = first tile row of each node
    size_by_node = [0] * nnodes
    for p in range(nnodes):
        size_by_node[(p + node_start) % nnodes] = sizes_by_pos[p]
    node_offset = sum(size_by_node[:nid])
    local_rank = rank % local_world
    if mode == "ag":
        tiled_m_start = cdiv(m_node * nid + m_r * local_rank, block_m)
    else:
        tiled_m_start = (m_node * nid + m_r * (local_rank + 1)) // block_m
    rank_offset = max(0, tiled_m_start - node_offset)
    intra = (tiled_m - offset_in_order + rank_offset) % tile_size
    return node_offset + intra


def ag_swizzle_multinode(tiled_m, m, rank, world, nnodes, block_m):
    """Tile-row permutation of AllGather-GEMM across nodes (Appendix "Swizzle", first
    listing): visit the own node's rows first, then the following nodes; inside a node
    start at the own local rank's rows."""
    return _multinode_swizzle(tiled_m, m, rank, world, nnodes, block_m, "ag")


def rs_swizzle_multinode(tiled_m, m, rank, world, nnodes, block_m):
    """Tile-row permutation of GEMM-ReduceScatter across nodes (Appendix "Swizzle", second
    listing): start with the next node's rows, and inside a node with the next local
    rank's rows."""
    return _multinode_swizzle(tiled_m, m, rank, world, nnodes, block_m, "rs")
