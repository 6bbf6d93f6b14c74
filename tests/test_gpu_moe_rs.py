"""MoE down-projection + ReduceScatter on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import moe as omoe, moe_rs as ors, gemm_rs as ogrs, formats, compare

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits  # noqa: E402


def _case(world, t_r, inter_r, hidden, experts, top_k, local, seed, integer):
    """Every rank's inputs: its own activations (rows in its gathered order) and down-projection weights."""
    rng = synth.rng_for(seed, 41, world)
    ids = synth.routing_topk(rng, world * t_r, experts, top_k)
    gen = (lambda shape, std: synth.integer_bf16(rng, shape, -2, 2)) if integer else \
        (lambda shape, std: synth.normal_bf16(rng, shape, std))
    hs, ws, e0s = [], [], []
    for r in range(world):
        e0 = (r * local) % experts if local < experts else 0
        _, offsets, gather = omoe.route(ids, world, experts, e0, local)
        hs.append(gen((int(offsets[-1]), inter_r), 1.0))
        ws.append(gen((local, inter_r, hidden), (inter_r * world) ** -0.5))
        e0s.append(e0)
    return ids, hs, ws, e0s


def _run(B, ids, hs, ws, e0s, d, world, t_r, inter_r, hidden, experts, top_k, local, chunks, gate, integer,
         flags=None, order=None, kn=False):
    _, offsets, gather = omoe.route(ids, world, experts, e0s[d], local)
    R = int(offsets[-1])
    max_rows = max(R, 1) + 7
    tokens = world * t_r
    # what the peers contribute: their own partials' rows for this rank (from the oracle's ordered arithmetic,
    # rounded to bf16 as a peer's combine would)
    peers = []
    for s in range(world):
        if s == d:
            peers.append(None)
            continue
        z = ors.partial(hs[s], ws[s], ids, world, experts, e0s[s], gate)
        peers.append(to_dev(formats.encode_bf16_rne(z[d * t_r:(d + 1) * t_r].astype(np.float32))))
    i32 = dict(dtype=torch.int32, device="cuda")
    y = torch.full((max_rows, hidden), 0x7FC0, dtype=torch.int16, device="cuda")
    inv = torch.full((tokens * top_k,), 12345, **i32)
    rec = torch.full((1 + 5 * B.moe_max_tiles(max_rows, local),), -1, **i32)
    combined = torch.full((tokens, hidden), 0x7FC0, dtype=torch.int16, device="cuda")
    scatter = torch.zeros((world, t_r, hidden), dtype=torch.int16, device="cuda")
    out = torch.full((t_r, hidden), 0x7FC0, dtype=torch.int16, device="cuda")
    signals = torch.zeros(B.signal_words(world, chunks), **i32)
    status = torch.zeros(B.STATUS_WORDS, **i32)
    if flags == B.FLAGS_PRESET:
        for s in range(world):
            if s != d:
                scatter[s].copy_(peers[s])
    w = ws[d] if kn else np.ascontiguousarray(np.transpose(ws[d], (0, 2, 1)))      # [E, hidden, inter] when B_NK
    st = B.moe_grouped_gemm_rs(to_dev(hs[d]) if R else torch.zeros((1, inter_r), dtype=torch.int16, device="cuda"),
                               to_dev(w), B.B_KN if kn else B.B_NK, None if gate is None else to_dev(gate.reshape(-1)),
                               to_dev(gather.astype(np.int32)) if R else torch.zeros(1, **i32), to_dev(offsets.astype(np.int32)),
                               y, inv, rec, combined, None if flags == B.FLAGS_PRESET else peers, scatter, out, signals, status,
                               order, t_r, hidden, inter_r, experts, top_k, local, max_rows, world, d, chunks, 3,
                               B.EMULATE_PRODUCER if flags is None else flags)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert status.cpu().tolist()[0] == 0
    # integer bookkeeping: the inverse index, bit for bit
    assert np.array_equal(inv.cpu().numpy(), ors.inverse_index(gather, tokens * top_k))
    # stage 1: the grouped GEMM
    y_ref = ors.down_proj(hs[d], ws[d], offsets)
    y_got = bits(y)
    if integer:
        assert np.array_equal(y_got[:R], formats.encode_bf16_rne(y_ref.astype(np.float32)))
    elif R:
        assert compare.max_row_rel_error(formats.decode_bf16(y_got[:R]), y_ref) <= TOL_BF16
    assert (y_got[R:] == 0x7FC0).all()
    # stage 2: the combine on what the GEMM produced: the specified fp32 order, bit for bit (gates here are
    # powers of two or absent, so the fused multiply-add is exact)
    z_got = bits(combined)
    assert np.array_equal(z_got, ors.combine_f32_ordered(y_got[:R], gather, tokens, top_k, gate))
    # stage 3: the reduction on the slots as they were: bit for bit; and the whole against the fp64 definition
    slots = [z_got[d * t_r:(d + 1) * t_r] if s == d else bits(peers[s]) for s in range(world)]
    assert np.array_equal(bits(out), ogrs.reduce_slots_f32_ordered(slots))
    ref = ors.moe_rs(hs, ws, ids, experts, e0s, d, gate)
    if integer and gate is None:
        assert np.array_equal(bits(out), formats.encode_bf16_rne(ref.astype(np.float32)))
    else:
        assert compare.max_row_rel_error(formats.decode_bf16(bits(out)), ref) <= 2 * TOL_BF16   # bf16 partials are rounded twice on the way
    sig = signals.cpu().numpy()
    if flags != B.FLAGS_PRESET:
        assert sig[2 * world:2 * world + world * chunks].tolist() == [3] * (world * chunks)      # every slot's chunks flagged
    assert not sig[:2 * world].any() and not sig[2 * world + world * chunks:].any()             # counters back at zero
    for s in range(world):
        if s != d:
            assert torch.equal(scatter[s], peers[s])


@pytest.mark.parametrize("world,t_r,inter_r,hidden,experts,top_k,local,chunks,integer", [
    (2, 64, 64, 128, 4, 2, 4, 1, True),           # every expert on every rank (the paper's placement)
    (4, 100, 72, 136, 12, 3, 12, 2, True),        # ragged contraction tail and width
    (8, 128, 192, 256, 32, 2, 32, 4, False),      # the table's expert count and top-k at 1/8 of its tokens
    (4, 96, 64, 264, 8, 2, 2, 3, True),           # experts sharded over the ranks: most assignments are elsewhere
    (1, 300, 64, 64, 3, 1, 3, 1, True),           # one rank: no peers
    (8, 256, 64, 1544, 8, 2, 8, 2, True),         # 4096 rows x 1544 columns: the 256-column block
])
def test_moe_rs_end_to_end(B, world, t_r, inter_r, hidden, experts, top_k, local, chunks, integer):
    ids, hs, ws, e0s = _case(world, t_r, inter_r, hidden, experts, top_k, local, seed=world, integer=integer)
    gate = None if integer else (2.0 ** synth.rng_for(3, 41, 7).integers(-2, 1, size=ids.shape)).astype(np.float32)
    for d in sorted({0, world - 1}):
        order = None if d == 0 else [s for s in range(world) if s != d]
        _run(B, ids, hs, ws, e0s, d, world, t_r, inter_r, hidden, experts, top_k, local, chunks, gate, integer, order=order)


def test_moe_rs_weights_kn_and_flags_preset(B):
    world, t_r, inter_r, hidden, experts, top_k = 4, 64, 72, 136, 6, 2
    ids, hs, ws, e0s = _case(world, t_r, inter_r, hidden, experts, top_k, experts, seed=5, integer=True)
    _run(B, ids, hs, ws, e0s, 1, world, t_r, inter_r, hidden, experts, top_k, experts, 2, None, True, kn=True)
    _run(B, ids, hs, ws, e0s, 2, world, t_r, inter_r, hidden, experts, top_k, experts, 2, None, True, flags=B.FLAGS_PRESET)


def test_moe_rs_large_experts_and_row_overflow(B):
    # 2048 rows per expert: the 256-row tile
    world, t_r, inter_r, hidden, experts, top_k = 8, 512, 128, 264, 4, 2
    ids, hs, ws, e0s = _case(world, t_r, inter_r, hidden, experts, top_k, experts, seed=6, integer=True)
    assert B.moe_tile_choice(world * t_r, top_k, experts, experts, hidden)[1] == 256
    _run(B, ids, hs, ws, e0s, 3, world, t_r, inter_r, hidden, experts, top_k, experts, 1, None, True)
    # more rows than the buffers hold: reported, no tile runs
    i32 = dict(dtype=torch.int32, device="cuda")
    fake16 = torch.zeros((64, 64), dtype=torch.int16, device="cuda")
    offsets = torch.tensor([0, 40, 90], **i32)
    status = torch.zeros(B.STATUS_WORDS, **i32)
    st = B.moe_grouped_gemm_rs(fake16, fake16, B.B_NK, None, torch.zeros(128, **i32), offsets, fake16, torch.zeros(128, **i32),
                               torch.zeros(1 + 5 * B.moe_max_tiles(64, 2), **i32), fake16, None, None, fake16,
                               torch.zeros(B.signal_words(1, 1), **i32), status, None, 64, 64, 64, 2, 2, 2, 64, 1, 0, 1, 1,
                               B.EMULATE_PRODUCER)
    assert st == B.OK
    torch.cuda.synchronize()
    s = status.cpu().tolist()
    assert s[0] == B.ERR_WORKSPACE and s[2] == 90
