"""MoE AllGather + grouped GEMM on the GPU against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import synth
from oracle import moe as omoe, formats, compare

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def B():
    from paper_2605_02953_amd import binding
    assert torch.cuda.is_available()
    return binding


from gpu_util import to_dev, bits, MoeRun  # noqa: E402


def w_nk(w_ekn):
    """logical [E_l, hidden, inter] -> physical [E_l, inter, hidden]."""
    return np.ascontiguousarray(np.transpose(w_ekn, (0, 2, 1)))


def _run_and_check(B, cfg, xs, ids, w, max_rows, integer, order=None, block_m=128, kn=False, tuning=None):
    st0, bm, bn = B.moe_tile_choice(cfg.world * cfg.tokens_per_rank, cfg.top_k, cfg.num_experts, cfg.num_local_experts, cfg.n)
    assert st0 == B.OK and bm == block_m and bn in (128, 192, 256)
    e0 = cfg.rank * cfg.num_local_experts if (cfg.rank + 1) * cfg.num_local_experts <= cfg.num_experts else 0
    run = MoeRun(B, cfg.world, cfg.tokens_per_rank, cfg.k, cfg.n, cfg.num_experts, cfg.top_k,
                 cfg.num_local_experts, max_rows)
    # kn: the weights handed over as they are stored logically, [E_l, hidden, inter]
    st = run([to_dev(x) for x in xs], to_dev(ids), to_dev(w if kn else w_nk(w)), e0, cfg.rank, order=order,
             w_layout=B.B_KN if kn else B.B_NK, tuning=tuning)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    assert run.status.cpu().tolist()[0] == 0
    # integer results: bit-exact
    count, offsets, gather = omoe.route(ids, cfg.world, cfg.num_experts, e0, cfg.num_local_experts)
    R = int(offsets[-1])
    assert np.array_equal(run.counts.cpu().numpy().reshape(cfg.world, cfg.num_experts), count)
    assert np.array_equal(run.offsets.cpu().numpy(), offsets)
    assert np.array_equal(run.gather.cpu().numpy()[:R], gather)
    assert (run.gather.cpu().numpy()[R:] == -1).all()
    sch = omoe.tile_schedule(count, e0, cfg.num_local_experts, block_m, cfg.rank, cfg.world)
    rec = run.records.cpu().numpy()
    assert rec[0] == sch["ntiles"]
    got = rec[1:1 + 4 * sch["ntiles"]].reshape(-1, 4)
    want = np.stack([sch["expert_id"], sch["tiled_m"], sch["segment_start"], sch["segment_end"]], axis=1) \
        if sch["ntiles"] else np.zeros((0, 4), dtype=np.int64)
    assert np.array_equal(got, want)
    # gathered tokens landed in the workspace unchanged
    assert np.array_equal(bits(run.workspace), np.concatenate(xs, axis=0))
    # floating point
    y = bits(run.y)
    ref = omoe.grouped_gemm(xs, ids, w, cfg.world, cfg.num_experts, e0)
    if integer:
        assert np.array_equal(y[:R], formats.encode_bf16_rne(ref.astype(np.float32)))
    else:
        assert compare.max_row_rel_error(formats.decode_bf16(y[:R]), ref) <= TOL_BF16
    assert (y[R:] == 0x7FC0).all()          # rows beyond R are not written
    return run, R


@pytest.mark.parametrize("world,t_r,hidden,inter,experts,top_k,local,rank,integer", [
    (2, 64, 64, 128, 4, 2, 2, 1, True),
    (4, 100, 72, 136, 12, 3, 3, 2, True),       # ragged hidden tail and width, odd expert counts
    (8, 128, 256, 264, 64, 2, 8, 5, True),
    (8, 128, 512, 384, 16, 2, 16, 3, False),    # every expert local (the paper's placement)
    (1, 300, 64, 64, 3, 1, 3, 0, True),
    (8, 256, 64, 1544, 8, 2, 8, 2, True),       # 4096 rows x 1544 columns: the 256-column block, ragged last block
    (8, 128, 64, 1400, 16, 2, 16, 6, True),     # 2048 rows x 1400 columns: the 192-column block, ragged last block
])
@pytest.mark.parametrize("kn", [False, True], ids=["w_nk", "w_kn"])
def test_moe_end_to_end(B, world, t_r, hidden, inter, experts, top_k, local, rank, integer, kn):
    cfg = synth.CONFIGS[4].scaled(world=world, tokens_per_rank=t_r, k=hidden, n=inter, num_experts=experts,
                                  top_k=top_k, num_local_experts=local, rank=rank)
    xs, ids, w = synth.moe_inputs(cfg, integer=integer)
    max_rows = world * t_r * top_k
    order = None if rank % 2 else list(reversed(range(world)))
    _run_and_check(B, cfg, xs, ids, w, max_rows, integer, order=order, kn=kn)


@pytest.mark.parametrize("hidden,inter,experts,top_k", [
    (2048, 176, 60, 4),      # Qwen1.5-MoE-A2.7B
    (14336, 512, 8, 2),      # Mixtral-8x7B
    (16384, 768, 8, 2),      # Mixtral-8x22B
    (1408, 256, 64, 6),      # DeepSeek-MoE
])
def test_moe_table_shapes_tensor_parallel_placement(B, hidden, inter, experts, top_k):
    """The paper's AllGather+MoE shapes (Appendix "Evaluation Setup", MoE shape table) in its own placement:
    every expert on every rank, the intermediate size divided by the 8 ranks; 8 x 128 tokens instead of
    8 x 1024 so that the oracle stays quick."""
    cfg = synth.CONFIGS[4].scaled(world=8, tokens_per_rank=128, k=hidden, n=inter, num_experts=experts,
                                  top_k=top_k, num_local_experts=experts, rank=0)
    xs, ids, w = synth.moe_inputs(cfg)
    _run_and_check(B, cfg, xs, ids, w, 8 * 128 * top_k, integer=False)


def test_moe_large_experts_use_the_256_row_tile(B):
    """2048 rows per expert (the Mixtral-8x22B shape at half its tokens): the schedule is cut in 256-row tiles."""
    cfg = synth.CONFIGS[4].scaled(world=8, tokens_per_rank=512, k=2048, n=776, num_experts=8, top_k=2,
                                  num_local_experts=8, rank=0)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    _run_and_check(B, cfg, xs, ids, w, 8 * 512 * 2, integer=True, block_m=256)
    _run_and_check(B, cfg, xs, ids, w, 8 * 512 * 2, integer=True, block_m=256, kn=True)


@pytest.mark.parametrize("groups", [1, 2, 3, 8])
@pytest.mark.parametrize("world,t_r,experts,top_k,local,rank", [
    (4, 100, 12, 3, 3, 2),        # 1200 assignments: most waves of eight work-groups have nothing to scan
    (8, 128, 64, 6, 64, 5),       # 6144 assignments over 64 local experts
    (8, 520, 60, 4, 60, 1),       # 16640 assignments: ranges that end inside a rank's shard
])
def test_moe_routing_shared_by_several_work_groups(B, groups, world, t_r, experts, top_k, local, rank):
    """counts, offsets, gather index and tile list do not depend on how many work-groups share the scan."""
    cfg = synth.CONFIGS[4].scaled(world=world, tokens_per_rank=t_r, k=64, n=128, num_experts=experts,
                                  top_k=top_k, num_local_experts=local, rank=rank)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    _run_and_check(B, cfg, xs, ids, w, world * t_r * top_k, True, tuning=B.tuning(moe_route_groups=groups))


def test_moe_route_groups_out_of_range_is_refused(B):
    cfg = synth.CONFIGS[4].scaled(world=2, tokens_per_rank=64, k=64, n=128, num_experts=2, top_k=1,
                                  num_local_experts=2, rank=0)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    run = MoeRun(B, 2, 64, 64, 128, 2, 1, 2, max_rows=128)
    st = run([to_dev(x) for x in xs], to_dev(ids), to_dev(w_nk(w)), 0, 0, tuning=B.tuning(moe_route_groups=9))
    assert st == B.ERR_INVALID_ARG


def test_moe_many_small_experts_use_the_256_row_tile_when_it_saves_a_round(B):
    """64 experts x 576 rows x 248 columns: 320 tiles of 128 rows (two rounds on 256 units) against 176 of 256 rows."""
    assert B.moe_tile_choice(8 * 768, 6, 64, 64, 248) == (B.OK, 256, 256)
    assert B.moe_tile_choice(8 * 512, 6, 64, 64, 248)[1] == 128      # 224 tiles of 128 rows: a single round either way
    cfg = synth.CONFIGS[4].scaled(world=8, tokens_per_rank=768, k=64, n=248, num_experts=64, top_k=6,
                                  num_local_experts=64, rank=3)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    _run_and_check(B, cfg, xs, ids, w, 8 * 768 * 6, integer=True, block_m=256)


def test_moe_degenerate_routings(B):
    cfg = synth.CONFIGS[4].scaled(world=4, tokens_per_rank=96, k=64, n=128, num_experts=8, top_k=1,
                                  num_local_experts=4, rank=1)
    xs, _, w = synth.moe_inputs(cfg, integer=True)
    # everything to one local expert; then nothing to any local expert
    for target in (5, 0):
        ids = np.full((4 * 96, 1), target, dtype=np.int32)
        _run_and_check(B, cfg, xs, ids, w, 4 * 96, True)


def test_moe_row_overflow_is_reported(B):
    cfg = synth.CONFIGS[4].scaled(world=2, tokens_per_rank=64, k=64, n=128, num_experts=2, top_k=1,
                                  num_local_experts=2, rank=0)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    run = MoeRun(B, 2, 64, 64, 128, 2, 1, 2, max_rows=100)          # 128 rows are routed here
    st = run([to_dev(x) for x in xs], to_dev(ids), to_dev(w_nk(w)), 0, 0)
    assert st == B.OK
    torch.cuda.synchronize()
    s = run.status.cpu().tolist()
    assert s[0] == B.ERR_WORKSPACE and s[2] == 128
    assert (bits(run.y) == 0x7FC0).all()


def test_cfg4_full_size(B):
    cfg = synth.CONFIGS[4]
    xs, ids, w = synth.moe_inputs(cfg)
    run, R = _run_and_check(B, cfg, xs, ids, w, max_rows=4096, integer=False)
    assert 1500 < R < 2600


def test_moe_expert_id_out_of_range_is_reported(B):
    """An id that names no expert is an error (the routing counts would no longer sum to tokens x top_k):
    status says which assignment, no tile runs, and the buffers are usable again afterwards."""
    cfg = synth.CONFIGS[4].scaled(world=4, tokens_per_rank=96, k=64, n=128, num_experts=8, top_k=2,
                                  num_local_experts=4, rank=1)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    run = MoeRun(B, 4, 96, 64, 128, 8, 2, 4, max_rows=4 * 96 * 2)
    xd, wd = [to_dev(x) for x in xs], to_dev(w_nk(w))
    for bad_value, where, groups in ((8, 301, 0), (-1, 17, 0), (8, 301, 3), (-1, 17, 8)):
        bad = ids.copy()
        bad.reshape(-1)[where] = bad_value
        bad.reshape(-1)[where + 200] = bad_value        # the smallest offending index is the one reported
        assert run(xd, to_dev(bad), wd, 4, 1, tuning=B.tuning(moe_route_groups=groups)) == B.OK
        torch.cuda.synchronize()
        s = run.status.cpu().tolist()
        assert s[0] == B.ERR_INVALID_ARG and s[1] == where
        assert run.records.cpu()[0] == 0 and (bits(run.y) == 0x7FC0).all()
        run.status.zero_()
    _run_and_check(B, cfg, xs, ids, w, 4 * 96 * 2, True)


def test_moe_flags_preset(B):
    """DITRON_FLAGS_PRESET: the gathered tokens are already in the workspace; nothing is copied, no flag is read."""
    cfg = synth.CONFIGS[4].scaled(world=4, tokens_per_rank=100, k=72, n=136, num_experts=12, top_k=3,
                                  num_local_experts=3, rank=2)
    xs, ids, w = synth.moe_inputs(cfg, integer=True)
    e0 = cfg.rank * cfg.num_local_experts
    run = MoeRun(B, 4, 100, 72, 136, 12, 3, 3, max_rows=1200)
    run.workspace.copy_(to_dev(np.concatenate(xs, axis=0)))
    assert run(None, to_dev(ids), to_dev(w_nk(w)), e0, cfg.rank, flags=B.FLAGS_PRESET) == B.OK
    torch.cuda.synchronize()
    # (the only words written are the flags of the routing work-groups, behind the 4 x world shard words)
    assert run.status.cpu().tolist()[0] == 0 and not run.signals[:4 * cfg.world].any()
    ref = omoe.grouped_gemm(xs, ids, w, cfg.world, cfg.num_experts, e0)
    assert np.array_equal(bits(run.y)[:ref.shape[0]], formats.encode_bf16_rne(ref.astype(np.float32)))
