"""ctypes binding of libditron.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors used purely as device memory; nothing here computes.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libditron.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_TIMEOUT = range(6)
BF16, FP8_E4M3 = 0, 1
B_KN, B_NK = 0, 1
EMULATE_PRODUCER, EXTERNAL_PRODUCER, FLAGS_PRESET, DUMP_SCHEDULE, DUMP_TIMING, EPOCH_IN_MEMORY = 1, 2, 4, 8, 16, 32
SCHEDULE_WORDS = 4
MAX_WORLD = 32
STATUS_WORDS = 4

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_02953_amd.build`")

lib = ctypes.CDLL(LIB_PATH)

_vp, _i, _u, _i32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_int32
_pp = ctypes.POINTER(ctypes.c_void_p)
_ip = ctypes.POINTER(ctypes.c_int)



class Tuning(ctypes.Structure):
    """ditron_tuning_t: per-call options; zero fields mean the defaults."""
    _fields_ = [("num_nodes", ctypes.c_int), ("spin_limit", ctypes.c_uint), ("decode_variant", ctypes.c_int),
                ("moe_route_groups", ctypes.c_int), ("reserved", ctypes.c_int * 4)]


_tp = ctypes.POINTER(Tuning)

lib.ditron_signal_words.restype = ctypes.c_size_t
lib.ditron_signal_words.argtypes = [_i, _i]
lib.ditron_ag_gemm_workspace_bytes.restype = ctypes.c_size_t
lib.ditron_ag_gemm_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i, _tp]
lib.ditron_moe_workspace_bytes.restype = ctypes.c_size_t
lib.ditron_moe_workspace_bytes.argtypes = [_i, _i, _i]
lib.ditron_schedule_dump.restype = _i
lib.ditron_schedule_dump.argtypes = [_i, _i, _i, _i, _i, _i, _i, _i, _tp, ctypes.POINTER(ctypes.c_int32), _i, _ip]
lib.ditron_tile_row_order.restype = _i
lib.ditron_tile_row_order.argtypes = [_i, _i, _i, _i, _i, _i, _ip]
lib.ditron_tile_config.restype = _i
lib.ditron_tile_config.argtypes = [_i, _i, _i, _i, _i, _tp, _ip]
lib.ditron_status_string.restype = ctypes.c_char_p
lib.ditron_status_string.argtypes = [_i]
lib.ditron_ag_gemm.restype = _i
lib.ditron_ag_gemm.argtypes = [_pp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _ip,
                               _i, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_ag_gemm_static.restype = _i
lib.ditron_ag_gemm_static.argtypes = [_pp, _vp, _i, _vp, _vp, _vp, _vp, _ip, _i, _i, _i, _i, _i, _i, _tp, _vp]
lib.ditron_gemm_rs.restype = _i
lib.ditron_gemm_rs.argtypes = [_vp, _vp, _i, _vp, _pp, _vp, _vp, _vp, _vp, _vp, _ip,
                               _i, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_gemm_rs_fuse_scatter.restype = _i
lib.ditron_gemm_rs_fuse_scatter.argtypes = [_vp, _vp, _i, _pp, _pp, _vp, _vp, _vp, _vp, _ip,
                                            _i, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_gemm_ar.restype = _i
lib.ditron_gemm_ar.argtypes = [_vp, _vp, _i, _vp, _pp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_gemm_ar_two_shot.restype = _i
lib.ditron_gemm_ar_two_shot.argtypes = [_vp, _vp, _i, _vp, _pp, _pp, _pp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_reduce_slots.restype = _i
lib.ditron_reduce_slots.argtypes = [_pp, _vp, _vp, _vp, _i, _i, _i, _i, _i32, _tp, _vp]
lib.ditron_moe_ag_grouped_gemm.restype = _i
lib.ditron_moe_ag_grouped_gemm.argtypes = [_pp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _ip,
                                           _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_moe_grouped_gemm_rs.restype = _i
lib.ditron_moe_grouped_gemm_rs.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _pp, _vp, _vp, _vp, _vp, _ip,
                                           _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i32, _u, _tp, _vp]
lib.ditron_moe_tile_choice.restype = _i
lib.ditron_moe_tile_choice.argtypes = [_i, _i, _i, _i, _i, _ip]
lib.ditron_moe_max_tiles.restype = _i
lib.ditron_moe_max_tiles.argtypes = [_i, _i]
lib.ditron_publish_chunks.restype = _i
lib.ditron_publish_chunks.argtypes = [_pp, _pp, ctypes.POINTER(ctypes.c_size_t), _ip, _vp, _i, _i32, _u, _vp]


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _ptr_array(tensors):
    if tensors is None:
        return None
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else (t if isinstance(t, int) else t.data_ptr())
    return arr


def _int_array(v):
    if v is None:
        return None
    return (ctypes.c_int * len(v))(*[int(x) for x in v])


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def status_string(code):
    return lib.ditron_status_string(int(code)).decode()


def signal_words(world, chunks=1):
    return int(lib.ditron_signal_words(world, chunks))


def tuning(num_nodes=0, spin_limit=0, decode_variant=0, moe_route_groups=0):
    """A ditron_tuning_t to pass as `tuning=`."""
    return Tuning(num_nodes, spin_limit, decode_variant, moe_route_groups)


def _tuning(t):
    return None if t is None else ctypes.byref(t)


def ag_gemm_workspace_bytes(m_per_rank, n, k, world, dtype=BF16, b_layout=B_NK, tuning=None):
    return int(lib.ditron_ag_gemm_workspace_bytes(m_per_rank, n, k, world, dtype, b_layout, _tuning(tuning)))


def moe_workspace_bytes(tokens_per_rank, hidden, world):
    return int(lib.ditron_moe_workspace_bytes(tokens_per_rank, hidden, world))


def schedule_dump(op, m, n, k, world, rank, dtype=BF16, b_layout=B_NK, tuning=None, capacity=None):
    """(status, records) with records a list of (pid_m, pid_n, first, last), one per GEMM work-group."""
    count = ctypes.c_int(0)
    if capacity is None:
        lib.ditron_schedule_dump(op, m, n, k, world, rank, dtype, b_layout, _tuning(tuning), None, 0, ctypes.byref(count))
        capacity = count.value
    out = (ctypes.c_int32 * max(1, SCHEDULE_WORDS * capacity))()
    st = lib.ditron_schedule_dump(op, m, n, k, world, rank, dtype, b_layout, _tuning(tuning), out, capacity,
                                  ctypes.byref(count))
    if st != OK:
        return st, []
    v = list(out)[:SCHEDULE_WORDS * count.value]
    return st, [tuple(v[i:i + SCHEDULE_WORDS]) for i in range(0, len(v), SCHEDULE_WORDS)]


def tile_row_order(op, m, block_m, world, nnodes, rank):
    npm = -(-m // block_m)
    out = (ctypes.c_int * npm)()
    st = lib.ditron_tile_row_order(op, m, block_m, world, nnodes, rank, out)
    return st, list(out)


def tile_config(op, m, n, k, dtype=BF16, tuning=None):
    out = (ctypes.c_int * 10)()
    st = lib.ditron_tile_config(op, m, n, k, dtype, _tuning(tuning), out)
    keys = ("block_m", "block_n", "group_m", "num_xcd", "per_xcd", "ntiles", "threads", "direct_staging", "splits")
    return st, dict(zip(keys, list(out)))


def ag_gemm(a_shards, b, b_layout, c, a_scales, b_scales, workspace, signals, status, schedule_out,
            arrival_order, m_per_rank, n, k, world, rank, dtype, epoch, flags, stream=None, tuning=None):
    return lib.ditron_ag_gemm(_ptr_array(a_shards), _ptr(b), b_layout, _ptr(c), _ptr(a_scales), _ptr(b_scales),
                              _ptr(workspace), _ptr(signals), _ptr(status), _ptr(schedule_out),
                              _int_array(arrival_order), m_per_rank, n, k, world, rank, dtype, epoch, flags,
                              _tuning(tuning), _stream(stream))


class PreparedAgGemm:
    """ditron_ag_gemm with its arguments marshalled once: for loops that call the same problem again and again
    and only advance the epoch (a ctypes call with ready-made arguments costs a few microseconds, building
    them every time about ten)."""

    def __init__(self, a_shards, b, b_layout, c, a_scales, b_scales, workspace, signals, status, schedule_out,
                 arrival_order, m_per_rank, n, k, world, rank, dtype, flags, stream=None, tuning=None):
        self._keep = (a_shards, b, c, a_scales, b_scales, workspace, signals, status, schedule_out, tuning)
        self._args = [_ptr_array(a_shards), _ptr(b), b_layout, _ptr(c), _ptr(a_scales), _ptr(b_scales), _ptr(workspace),
                      _ptr(signals), _ptr(status), _ptr(schedule_out), _int_array(arrival_order), m_per_rank, n, k,
                      world, rank, dtype, 0, flags, _tuning(tuning), _stream(stream)]

    def __call__(self, epoch):
        a = self._args
        a[17] = epoch
        return lib.ditron_ag_gemm(*a)


STATIC_WORKSPACE_BYTES = 32 << 20
MOE_ROUTE_SCRATCH_BYTES = 266240


def ag_gemm_static(a_shards, b, b_layout, c, a_scales, b_scales, status, arrival_order, m_per_rank, n, k, world,
                   rank, dtype, stream=None, tuning=None):
    return lib.ditron_ag_gemm_static(_ptr_array(a_shards), _ptr(b), b_layout, _ptr(c), _ptr(a_scales), _ptr(b_scales),
                                     _ptr(status), _int_array(arrival_order), m_per_rank, n, k, world, rank, dtype,
                                     _tuning(tuning), _stream(stream))


def gemm_rs(a, b, b_layout, gemm_out, peer_partials, scatter_buf, out, signals, status, schedule_out,
            arrival_order, m, n, k_local, world, rank, chunks_per_slot, epoch, flags, stream=None, tuning=None):
    return lib.ditron_gemm_rs(_ptr(a), _ptr(b), b_layout, _ptr(gemm_out), _ptr_array(peer_partials),
                              _ptr(scatter_buf), _ptr(out), _ptr(signals), _ptr(status), _ptr(schedule_out),
                              _int_array(arrival_order), m, n, k_local, world, rank, chunks_per_slot, epoch,
                              flags, _tuning(tuning), _stream(stream))


def gemm_rs_fuse_scatter(a, b, b_layout, scatter_dsts, peer_partials, out, signals, status, schedule_out,
                         arrival_order, m, n, k_local, world, rank, chunks_per_slot, epoch, flags, stream=None, tuning=None):
    return lib.ditron_gemm_rs_fuse_scatter(_ptr(a), _ptr(b), b_layout, _ptr_array(scatter_dsts),
                                           _ptr_array(peer_partials), _ptr(out), _ptr(signals), _ptr(status),
                                           _ptr(schedule_out), _int_array(arrival_order), m, n, k_local, world, rank,
                                           chunks_per_slot, epoch, flags, _tuning(tuning), _stream(stream))


def gemm_ar(a, b, b_layout, gemm_out, peer_partials, out, signals, status, schedule_out, m, n, k_local, world,
            rank, epoch, flags, stream=None, tuning=None):
    return lib.ditron_gemm_ar(_ptr(a), _ptr(b), b_layout, _ptr(gemm_out), _ptr_array(peer_partials), _ptr(out),
                              _ptr(signals), _ptr(status), _ptr(schedule_out), m, n, k_local, world, rank, epoch,
                              flags, _tuning(tuning), _stream(stream))


def gemm_ar_two_shot(a, b, b_layout, gemm_out, peer_partials, out_dsts, peer_reduced, signals, status, schedule_out,
                     m, n, k_local, world, rank, epoch, flags, stream=None, tuning=None):
    return lib.ditron_gemm_ar_two_shot(_ptr(a), _ptr(b), b_layout, _ptr(gemm_out), _ptr_array(peer_partials),
                                       _ptr_array(out_dsts), _ptr_array(peer_reduced), _ptr(signals), _ptr(status),
                                       _ptr(schedule_out), m, n, k_local, world, rank, epoch, flags, _tuning(tuning), _stream(stream))


def reduce_slots(slots, out, signals, status, rows, n, world, chunks, epoch, stream=None, tuning=None):
    return lib.ditron_reduce_slots(_ptr_array(slots), _ptr(out), _ptr(signals), _ptr(status), rows, n, world,
                                   chunks, epoch, _tuning(tuning), _stream(stream))


def moe_tile_choice(total_tokens, top_k, num_experts, num_local_experts, inter):
    out = (ctypes.c_int * 2)()
    st = lib.ditron_moe_tile_choice(total_tokens, top_k, num_experts, num_local_experts, inter, out)
    return st, out[0], out[1]


def moe_max_tiles(max_rows, num_local_experts):
    return int(lib.ditron_moe_max_tiles(max_rows, num_local_experts))


def moe_ag_grouped_gemm(x_shards, topk_ids, w, w_layout, y, counts, expert_offsets, gather_idx, tile_records,
                        workspace, signals, status, arrival_order, tokens_per_rank, hidden, inter, num_experts,
                        top_k, expert_begin, num_local_experts, max_rows, world, rank, epoch, flags, stream=None, tuning=None):
    return lib.ditron_moe_ag_grouped_gemm(_ptr_array(x_shards), _ptr(topk_ids), _ptr(w), w_layout, _ptr(y),
                                          _ptr(counts), _ptr(expert_offsets), _ptr(gather_idx),
                                          _ptr(tile_records), _ptr(workspace), _ptr(signals), _ptr(status),
                                          _int_array(arrival_order), tokens_per_rank, hidden, inter,
                                          num_experts, top_k, expert_begin, num_local_experts, max_rows, world,
                                          rank, epoch, flags, _tuning(tuning), _stream(stream))


def moe_grouped_gemm_rs(h, w, w_layout, topk_weights, gather_idx, expert_offsets, y, inverse_idx, tile_records, combined,
                        peer_partials, scatter_buf, out, signals, status, arrival_order, tokens_per_rank, hidden, inter,
                        num_experts, top_k, num_local_experts, max_rows, world, rank, chunks_per_slot, epoch, flags,
                        stream=None, tuning=None):
    return lib.ditron_moe_grouped_gemm_rs(_ptr(h), _ptr(w), w_layout, _ptr(topk_weights), _ptr(gather_idx),
                                          _ptr(expert_offsets), _ptr(y), _ptr(inverse_idx), _ptr(tile_records),
                                          _ptr(combined), _ptr_array(peer_partials), _ptr(scatter_buf), _ptr(out),
                                          _ptr(signals), _ptr(status), _int_array(arrival_order), tokens_per_rank,
                                          hidden, inter, num_experts, top_k, num_local_experts, max_rows, world, rank,
                                          chunks_per_slot, epoch, flags, _tuning(tuning), _stream(stream))


def publish_chunks(dst, src, nbytes, flag_index, signals, epoch, delay_cycles=0, stream=None):
    n = len(dst)
    sizes = (ctypes.c_size_t * n)(*[int(x) for x in nbytes])
    return lib.ditron_publish_chunks(_ptr_array(dst), _ptr_array(src), sizes, _int_array(flag_index),
                                     _ptr(signals), n, epoch, delay_cycles, _stream(stream))
