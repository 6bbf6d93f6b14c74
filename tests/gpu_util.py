"""Helpers for the GPU parity tests: move raw storage to the device, run one entry point
through the C ABI, bring raw storage back.  No arithmetic happens here."""
import numpy as np
import torch


def to_dev(arr):
    """numpy raw storage (uint16 bf16 bits / uint8 fp8 bytes / int32 / float32) -> device tensor."""
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def bits(t):
    """device tensor of bf16 storage (int16) -> numpy uint16."""
    return t.cpu().numpy().view(np.uint16)


def nk(b_kn):
    """logical [k, n] storage -> physical [n, k] (k contiguous)."""
    return np.ascontiguousarray(b_kn.T)


class AgGemmRun:
    """Buffers for repeated ditron_ag_gemm calls on one problem shape."""

    def __init__(self, B, world, m_per_rank, n, k, esize=2, b_layout=None, tuning=None):
        self.B, self.world, self.m_per_rank, self.n, self.k = B, world, m_per_rank, n, k
        m = world * m_per_rank
        dt = torch.int16 if esize == 2 else torch.uint8
        # the library says how large the workspace is; it starts with the gathered operand
        nbytes = B.ag_gemm_workspace_bytes(m_per_rank, n, k, world, B.BF16 if esize == 2 else B.FP8_E4M3,
                                           B.B_NK if b_layout is None else b_layout, tuning)
        assert nbytes >= m * k * esize
        self.ws_raw = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        self.workspace = self.ws_raw[:m * k * esize].view(dt).view(m, k)
        self.tuning = tuning
        self.c = torch.zeros((m, n), dtype=torch.int16, device="cuda")
        self.signals = torch.zeros(B.signal_words(world, 1), dtype=torch.int32, device="cuda")
        self.status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
        self.epoch = 0

    def __call__(self, shards_dev, b_dev, rank, order=None, flags=None, schedule=None, b_layout=None,
                 dtype=None, a_scales=None, b_scales=None, stream=None, tuning=None):
        B = self.B
        self.epoch += 1
        flags = B.EMULATE_PRODUCER if flags is None else flags
        if schedule is not None:
            flags |= B.DUMP_SCHEDULE
        st = B.ag_gemm(shards_dev, b_dev, B.B_NK if b_layout is None else b_layout, self.c, a_scales, b_scales,
                       self.ws_raw, self.signals, self.status, schedule, order, self.m_per_rank, self.n,
                       self.k, self.world, rank, B.BF16 if dtype is None else dtype, self.epoch, flags, stream,
                       self.tuning if tuning is None else tuning)
        return st


class GemmRsRun:
    """Buffers for repeated ditron_gemm_rs calls on one problem shape."""

    def __init__(self, B, world, m, n, k, chunks=1):
        self.B, self.world, self.m, self.n, self.k, self.chunks = B, world, m, n, k, chunks
        m_r = m // world
        self.gemm_out = torch.zeros((m, n), dtype=torch.int16, device="cuda")
        self.scatter = torch.zeros((world, m_r, n), dtype=torch.int16, device="cuda")
        self.out = torch.zeros((m_r, n), dtype=torch.int16, device="cuda")
        self.signals = torch.zeros(B.signal_words(world, chunks), dtype=torch.int32, device="cuda")
        self.status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
        self.epoch = 0

    def __call__(self, a_dev, b_dev, peers, rank, order=None, flags=None, schedule=None, stream=None, b_layout=None, tuning=None):
        B = self.B
        self.epoch += 1
        flags = B.EMULATE_PRODUCER if flags is None else flags
        if schedule is not None:
            flags |= B.DUMP_SCHEDULE
        return B.gemm_rs(a_dev, b_dev, B.B_NK if b_layout is None else b_layout, self.gemm_out, peers, self.scatter, self.out, self.signals,
                         self.status, schedule, order, self.m, self.n, self.k, self.world, rank, self.chunks,
                         self.epoch, flags, stream, tuning)


class MoeRun:
    """Buffers for repeated ditron_moe_ag_grouped_gemm calls on one problem shape."""

    def __init__(self, B, world, tokens_per_rank, hidden, inter, num_experts, top_k, num_local, max_rows):
        self.B = B
        self.dims = (tokens_per_rank, hidden, inter, num_experts, top_k, num_local, max_rows, world)
        self.max_tiles = B.moe_max_tiles(max_rows, num_local)
        i32 = dict(dtype=torch.int32, device="cuda")
        # the gathered tokens, then the routing work-groups' scratch, which needs no initialisation: fill it with a
        # pattern so that nothing can rely on zeros
        gathered = world * tokens_per_rank * hidden * 2
        self.ws_raw = torch.full((B.moe_workspace_bytes(tokens_per_rank, hidden, world),), 0x5A, dtype=torch.uint8, device="cuda")
        self.ws_raw[:gathered].zero_()
        self.workspace = self.ws_raw[:gathered].view(torch.int16).view(world * tokens_per_rank, hidden)
        self.y = torch.full((max_rows, inter), 0x7FC0, dtype=torch.int16, device="cuda")   # NaN pattern: untouched rows stay visible
        self.counts = torch.full((world * num_experts,), -1, **i32)
        self.offsets = torch.full((num_local + 1,), -1, **i32)
        self.gather = torch.full((max_rows,), -1, **i32)
        self.records = torch.full((1 + 5 * self.max_tiles,), -1, **i32)
        self.signals = torch.zeros(B.signal_words(world, 1), **i32)
        self.status = torch.zeros(B.STATUS_WORDS, **i32)
        self.epoch = 0

    def __call__(self, x_dev, ids_dev, w_dev, expert_begin, rank, order=None, flags=None, stream=None, w_layout=None, tuning=None):
        B = self.B
        t_r, hidden, inter, ne, top_k, nl, max_rows, world = self.dims
        self.epoch += 1
        flags = B.EMULATE_PRODUCER if flags is None else flags
        return B.moe_ag_grouped_gemm(x_dev, ids_dev, w_dev, B.B_NK if w_layout is None else w_layout, self.y, self.counts, self.offsets, self.gather,
                                     self.records, self.workspace, self.signals, self.status, order, t_r, hidden,
                                     inter, ne, top_k, expert_begin, nl, max_rows, world, rank, self.epoch, flags,
                                     stream, tuning)


class GemmArRun:
    """Buffers for repeated ditron_gemm_ar calls on one problem shape."""

    def __init__(self, B, world, m, n, k):
        self.B, self.world, self.m, self.n, self.k = B, world, m, n, k
        st, self.tc = B.tile_config(3, m, n, k)
        assert st == B.OK
        self.ntiles = self.tc["ntiles"]
        self.npn = -(-n // self.tc["block_n"])
        self.gemm_out = torch.zeros((m, n), dtype=torch.int16, device="cuda")
        self.out = torch.full((m, n), 0x7FC0, dtype=torch.int16, device="cuda")   # NaN pattern: unwritten output stays visible
        self.signals = torch.zeros(B.signal_words(world, self.ntiles), dtype=torch.int32, device="cuda")
        self.status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
        self.epoch = 0

    def flag_index(self, s, pid_m, pid_n):
        return 2 * self.world + s * self.ntiles + pid_m * self.npn + pid_n

    def __call__(self, a_dev, b_dev, peers, rank, flags=None, schedule=None, stream=None, b_layout=None, tuning=None):
        B = self.B
        self.epoch += 1
        flags = B.EMULATE_PRODUCER if flags is None else flags
        if schedule is not None:
            flags |= B.DUMP_SCHEDULE
        return B.gemm_ar(a_dev, b_dev, B.B_NK if b_layout is None else b_layout, self.gemm_out, peers, self.out,
                         self.signals, self.status, schedule, self.m, self.n, self.k, self.world, rank, self.epoch,
                         flags, stream, tuning)
