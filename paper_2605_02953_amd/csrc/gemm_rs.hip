// GEMM-ReduceScatter, one rank's share (paper, Appendix "GEMM Reduce-Scatter").
//
// Launch 1 holds the GEMM and the emulated peers.  The last `num_producers` work-groups
// copy, peer by peer in delivery order and row chunk by row chunk, the block each peer would
// push into this rank's scatter buffer, raising one flag per (peer, chunk).  The first
// work-groups are the tiles of the local GEMM P = A . B, visited from the segment of rank+1
// to the rank's own segment; a tile bumps the counter of every segment it touches and the
// tile that completes a segment raises the segment flag.
// Launch 2 is the reduction: each work-group waits for the flags of the row chunk it sums
// (the peers' arrival flags and the GEMM's flag for the own segment), adds the `world`
// blocks in fp32 in slot order with 128-bit loads, rounds once to bf16.
#include "gemm_core.h"
#include "launch.h"

namespace ditron {

struct GemmRsParams {
  const void* peer[DITRON_MAX_WORLD];
  int order[DITRON_MAX_WORLD];
  const char* a;
  const char* b;
  __bf16* gemm_out;
  __bf16* dst[DITRON_MAX_WORLD];   // fused scatter: rank d's [world, m_per_rank, n] buffer (dst[rank] is the local one)
  int fuse_scatter;
  char* scatter_buf;
  int32_t* seg_flags;      // [world]
  int32_t* seg_counters;   // [world]
  int32_t* arr_flags;      // [world * chunks]
  int32_t* arr_counters;   // [world * chunks]
  int32_t* status;
  int32_t* schedule;
  int m, n, k, world, rank, nnodes, m_per_rank, chunks, n_peers;
  int32_t epoch;
  int num_producers, teams;
  TileOrder tiling;
};

template <class T>
__global__ __launch_bounds__(T::THREADS) void gemm_rs_kernel(const GemmRsParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int ntiles = p.tiling.npm * p.tiling.npn;
  if ((int)blockIdx.x >= ntiles) {
    // The emulated peers sit behind the GEMM tiles in the grid: nothing in this launch waits for
    // them (only the reduction does), so they fill compute units as the last tiles drain instead
    // of taking units away from the GEMM's first wave.
    const int part = blockIdx.x - ntiles;
    const size_t slot_bytes = (size_t)p.m_per_rank * p.n * 2;
    const size_t chunk_bytes = slot_bytes / p.chunks;
    // chunk index i = (delivery position of the peer) * chunks + row chunk
    produce_chunks<T::THREADS>(
        p.n_peers * p.chunks, chunk_bytes, part, p.num_producers, p.teams, p.epoch,
        [&](int i) { return (void*)(p.scatter_buf + p.order[i / p.chunks] * slot_bytes + (i % p.chunks) * chunk_bytes); },
        [&](int i) { return (const void*)((const char*)p.peer[p.order[i / p.chunks]] + (i % p.chunks) * chunk_bytes); },
        [&](int i) { return p.arr_flags + p.order[i / p.chunks] * p.chunks + i % p.chunks; },
        [&](int i) { return p.arr_counters + p.order[i / p.chunks] * p.chunks + i % p.chunks; });
    return;
  }
  const int wg = blockIdx.x;
  const TileSpan t = tile_of_workgroup(wg, p.tiling, kOrderScatter, p.m, p.m_per_rank, p.rank, p.world, p.nnodes, T::BM);
  const int m0 = t.pid_m * T::BM, n0 = t.pid_n * T::BN;
  const int seg_start = t.first, seg_end = t.last;
  if (p.schedule && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * (size_t)wg;
    rec[0] = t.pid_m; rec[1] = t.pid_n; rec[2] = seg_start; rec[3] = seg_end;
  }
  const uint32_t row_bytes = (uint32_t)p.k * 2u;
  const int M = p.m, N = p.n;
  auto a_row = [=](int r) { return (uint32_t)min(m0 + r, M - 1) * row_bytes; };
  typename T::Acc acc;
  if constexpr (T::B_KN) {
    gemm_mainloop<T>(acc, p.a, a_row, p.b, BColumns{(uint32_t)N * 2u, n0, N}, p.k, lds);
  } else {
    auto b_row = [=](int r) { return (uint32_t)min(n0 + r, N - 1) * row_bytes; };
    gemm_mainloop<T>(acc, p.a, a_row, p.b, b_row, p.k, lds);
  }
  // streaming stores: the segment counter's release below would otherwise write the tile back out of the
  // chiplet's L2, and the partial is read only by the reduction, later (measured: 1.7 % of the step)
  if (p.fuse_scatter) {
    // the rows of segment d go straight to slot `rank` of rank d's buffer, row m landing at
    // rank * m_per_rank + m % m_per_rank (the listing's remote store)
    park_tile_bf16<T>(acc, lds);
    for (int seg = seg_start; seg <= seg_end; ++seg) {
      __bf16* c = p.dst[seg] + (ptrdiff_t)(p.rank - seg) * p.m_per_rank * p.n;
      store_parked_bf16<T, true>(c, (size_t)p.n, m0, n0, max(m0, seg * p.m_per_rank),
                                 min(min(m0 + T::BM, M), (seg + 1) * p.m_per_rank), N, lds);
    }
  } else {
    store_tile_bf16<T, true>(acc, p.gemm_out, (size_t)p.n, m0, n0, M, N, lds);
  }

  // segment completion: one lane per touched segment
  __syncthreads();
  const int seg = seg_start + (int)threadIdx.x;
  if (seg <= seg_end) {
    const int first = (p.m_per_rank * seg) / T::BM;
    const int last = (p.m_per_rank * (seg + 1) - 1) / T::BM;
    const int target = p.tiling.npn * (last - first + 1);
    // release-only arrivals; the tile that completes the segment adds the acquire (see publish_after_all)
    const int old = __hip_atomic_fetch_add(p.seg_counters + seg, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    if (old == target - 1) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(p.seg_counters + seg, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      flag_raise(p.seg_flags + seg, p.epoch);
    }
  }
}

// ------------------------------------------------------------------ reduction
struct ReduceParams {
  const void* slot[DITRON_MAX_WORLD];
  const int32_t* gate[DITRON_MAX_WORLD];  // first flag of slot s (chunk c at gate[s] + c*gate_stride[s]) or null
  int gate_stride[DITRON_MAX_WORLD];
  __bf16* out;
  int32_t* status;
  size_t vec_per_chunk;  // 16-byte vectors per row chunk
  int chunks, world;
  int32_t epoch;
  unsigned spin_limit;
  int wgs_per_chunk;
};

constexpr int kReduceThreads = 1024;
constexpr int kReduceUnroll = 1;     // 16-byte vectors per lane per slot in flight
constexpr int kReduceMaxWgs = 1024;

__device__ __forceinline__ void set_bf16x8(float (&acc)[8], const u32x4_t v) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] = __builtin_bit_cast(float, v[j] << 16);
    acc[2 * j + 1] = __builtin_bit_cast(float, v[j] & 0xFFFF0000u);
  }
}

__device__ __forceinline__ void add_bf16x8(float (&acc)[8], const u32x4_t v) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] += __builtin_bit_cast(float, v[j] << 16);
    acc[2 * j + 1] += __builtin_bit_cast(float, v[j] & 0xFFFF0000u);
  }
}

__device__ __forceinline__ u32x4_t pack_bf16x8(const float (&acc)[8]) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  u32x4_t r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    bf16x2_t v = {(__bf16)acc[2 * j], (__bf16)acc[2 * j + 1]};
    r[j] = __builtin_bit_cast(uint32_t, v);
  }
  return r;
}

// WORLD > 0 fixes the number of slots at compile time (fully unrolled slot loop).
template <int WORLD>
__global__ __launch_bounds__(kReduceThreads) void reduce_slots_kernel(const ReduceParams p) {
  const int chunk = blockIdx.x / p.wgs_per_chunk;
  const int part = blockIdx.x % p.wgs_per_chunk;
  const int world = WORLD > 0 ? WORLD : p.world;
  // one lane per slot: the flags are looked at side by side, not one round trip after another
  if ((int)threadIdx.x < world && p.gate[threadIdx.x])
    flag_wait_lane(p.gate[threadIdx.x], chunk * p.gate_stride[threadIdx.x], 1, p.epoch, p.spin_limit, p.status);
  __syncthreads();
  const size_t base = (size_t)chunk * p.vec_per_chunk;
  const size_t step = (size_t)p.wgs_per_chunk * kReduceThreads;
  u32x4_t* out = (u32x4_t*)p.out + base;
  size_t i = (size_t)part * kReduceThreads + threadIdx.x;
  for (; i + (kReduceUnroll - 1) * step < p.vec_per_chunk; i += kReduceUnroll * step) {
    float acc[kReduceUnroll][8];
    {
      u32x4_t v[kReduceUnroll];
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u)
        v[u] = __builtin_nontemporal_load((const u32x4_t*)p.slot[0] + base + i + u * step);
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u) set_bf16x8(acc[u], v[u]);
    }
#pragma unroll
    for (int s = 1; s < world; ++s) {
      u32x4_t v[kReduceUnroll];
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u)
        v[u] = __builtin_nontemporal_load((const u32x4_t*)p.slot[s] + base + i + u * step);
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u) add_bf16x8(acc[u], v[u]);
    }
#pragma unroll
    for (int u = 0; u < kReduceUnroll; ++u) __builtin_nontemporal_store(pack_bf16x8(acc[u]), out + i + u * step);
  }
  for (; i < p.vec_per_chunk; i += step) {
    float acc[8];
    set_bf16x8(acc, ((const u32x4_t*)p.slot[0])[base + i]);
    for (int s = 1; s < world; ++s) add_bf16x8(acc, ((const u32x4_t*)p.slot[s])[base + i]);
    out[i] = pack_bf16x8(acc);
  }
}

// `flags_pending`: some gate may still be down when the kernel starts (an external producer
// that needs room on the chip to run); the waiting work-groups are then kept to half the chip.
static ditron_status_t launch_reduce(ReduceParams& p, bool flags_pending, hipStream_t stream) {
  // enough work-groups to cover the chip several times over, at least one per row chunk
  const size_t per_wg = (size_t)kReduceThreads * kReduceUnroll;
  size_t want = (p.vec_per_chunk + per_wg - 1) / per_wg;
  bool gated = false;
  for (int s = 0; s < p.world; ++s) gated = gated || p.gate[s] != nullptr;
  const int max_wgs = (gated && flags_pending) ? 256 : kReduceMaxWgs;
  const size_t cap = (size_t)(max_wgs / p.chunks > 0 ? max_wgs / p.chunks : 1);
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  p.wgs_per_chunk = (int)want;
  const dim3 grid((unsigned)(p.wgs_per_chunk * p.chunks));
  if (p.world == 8) hipLaunchKernelGGL(reduce_slots_kernel<8>, grid, dim3(kReduceThreads), 0, stream, p);
  else if (p.world == 4) hipLaunchKernelGGL(reduce_slots_kernel<4>, grid, dim3(kReduceThreads), 0, stream, p);
  else if (p.world == 2) hipLaunchKernelGGL(reduce_slots_kernel<2>, grid, dim3(kReduceThreads), 0, stream, p);
  else hipLaunchKernelGGL(reduce_slots_kernel<0>, grid, dim3(kReduceThreads), 0, stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

template <class T>
static ditron_status_t launch_rs(GemmRsParams& p, hipStream_t stream) {
  p.tiling.npm = cdiv(p.m, T::BM);
  p.tiling.npn = cdiv(p.n, T::BN);
  if (!set_dynamic_lds<gemm_rs_kernel<T>>(T::LDS_BYTES)) return DITRON_ERR_HIP;
  const unsigned grid = (unsigned)(p.num_producers + p.tiling.npm * p.tiling.npn);
  hipLaunchKernelGGL(gemm_rs_kernel<T>, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

}  // namespace ditron

using namespace ditron;

extern "C" ditron_status_t ditron_reduce_slots(const void* const* slots, void* out, const int32_t* signals,
                                               int32_t* status, int rows, int n, int world, int chunks,
                                               int32_t epoch, const ditron_tuning_t* tuning, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rows <= 0 || n <= 0 || chunks < 1) return DITRON_ERR_INVALID_ARG;
  const Tuning tune = resolve_tuning(tuning, 1);
  if (!tune.valid) return DITRON_ERR_INVALID_ARG;
  if (!slots || !out || !aligned16(out) || (signals && !status)) return DITRON_ERR_INVALID_ARG;
  if (n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (rows % chunks != 0) return DITRON_ERR_INVALID_ARG;
  ReduceParams p{};
  for (int s = 0; s < world; ++s) {
    if (!slots[s] || !aligned16(slots[s])) return DITRON_ERR_INVALID_ARG;
    p.slot[s] = slots[s];
    p.gate[s] = signals ? signals + (size_t)s * chunks : nullptr;
    p.gate_stride[s] = 1;
  }
  p.out = (__bf16*)out;
  p.status = status;
  p.vec_per_chunk = (size_t)(rows / chunks) * n / 8;
  p.chunks = chunks;
  p.world = world;
  p.epoch = epoch;
  p.spin_limit = tune.spin_limit;
  return launch_reduce(p, /*flags_pending=*/signals != nullptr, (hipStream_t)stream);
}

static ditron_status_t gemm_rs_impl(const void* a, const void* b, int b_layout, void* gemm_out,
                                    void* const* scatter_dsts, const void* const* peer_partials, void* scatter_buf,
                                    void* out, int32_t* signals, int32_t* status, int32_t* schedule_out,
                                    const int* arrival_order, int m, int n, int k_local, int world, int rank,
                                    int chunks_per_slot, int32_t epoch, unsigned flags,
                                    const ditron_tuning_t* tuning, void* stream) {
  const bool fuse = scatter_dsts != nullptr;

  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (m <= 0 || n <= 0 || k_local <= 0 || m % world != 0 || chunks_per_slot < 1) return DITRON_ERR_INVALID_ARG;
  const Tuning tune = resolve_tuning(tuning, world);
  if (!tune.valid) return DITRON_ERR_INVALID_ARG;
  const int m_r = m / world;
  if (m_r % chunks_per_slot != 0) return DITRON_ERR_INVALID_ARG;
  if (!a || !b || (!fuse && !gemm_out) || !out || !signals || !status) return DITRON_ERR_INVALID_ARG;
  if (world > 1 && !scatter_buf) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(a) || !aligned16(b) || !aligned16(gemm_out) || !aligned16(out) || !aligned16(scatter_buf) ||
      !aligned16(signals))
    return DITRON_ERR_INVALID_ARG;
  const Mode mode = producer_mode(flags);
  if (flags & DITRON_EPOCH_IN_MEMORY) return DITRON_ERR_UNSUPPORTED;
  if (mode == Mode::kInvalid) return DITRON_ERR_INVALID_ARG;
  const bool emulate = mode == Mode::kEmulate;
  if ((flags & DITRON_DUMP_SCHEDULE) && !schedule_out) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (k_local % 8 != 0 || n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit(m, k_local, 2) || !fits_32bit(n, k_local, 2)) return DITRON_ERR_UNSUPPORTED;

  GemmRsParams p{};
  p.n_peers = world - 1;
  if (emulate) {
    if (world > 1 && !peer_partials) return DITRON_ERR_INVALID_ARG;
    bool seen[DITRON_MAX_WORLD] = {false};
    for (int i = 0; i < world - 1; ++i) {
      const int s = arrival_order ? arrival_order[i] : ((rank - 1 - i) % world + world) % world;
      if (s < 0 || s >= world || s == rank || seen[s]) return DITRON_ERR_INVALID_ARG;
      seen[s] = true;
      p.order[i] = s;
      if (!peer_partials[s] || !aligned16(peer_partials[s])) return DITRON_ERR_INVALID_ARG;
      p.peer[s] = peer_partials[s];
    }
  }
  p.a = (const char*)a;
  p.b = (const char*)b;
  p.gemm_out = (__bf16*)gemm_out;
  p.fuse_scatter = fuse;
  if (fuse) {
    for (int d = 0; d < world; ++d) {
      if (!scatter_dsts[d] || !aligned16(scatter_dsts[d])) return DITRON_ERR_INVALID_ARG;
      p.dst[d] = (__bf16*)scatter_dsts[d];
    }
  }
  p.scatter_buf = (char*)scatter_buf;
  p.seg_flags = signals;
  p.seg_counters = signals + world;
  p.arr_flags = signals + 2 * world;
  p.arr_counters = signals + 2 * world + world * chunks_per_slot;
  p.status = status;
  p.schedule = (flags & DITRON_DUMP_SCHEDULE) ? schedule_out : nullptr;
  p.m = m;
  p.n = n;
  p.k = k_local;
  p.world = world;
  p.rank = rank;
  p.nnodes = tune.num_nodes;
  p.m_per_rank = m_r;
  p.chunks = chunks_per_slot;
  p.epoch = epoch;
  TileChoice tc = choose_tile(m, n, k_local);
  if (p.nnodes > 1 && !node_order_is_bijection(m, tc.block_m, world, p.nnodes, rank, kOrderScatter))
    return DITRON_ERR_UNSUPPORTED;
  p.tiling.group_m = tc.group_m;
  p.tiling.num_xcd = tc.num_xcd;
  p.tiling.per_xcd = tc.per_xcd;
  const ProducerPlan pl = plan_producers((size_t)(world - 1) * m_r * n * 2, (world - 1) * chunks_per_slot);
  p.num_producers = (emulate && world > 1) ? pl.producers : 0;
  p.teams = pl.teams;
  ditron_status_t st;
  if (b_layout == DITRON_B_KN) {
    st = tc.big ? launch_rs<TileBigKN>(p, (hipStream_t)stream) : launch_rs<TileSmallKN>(p, (hipStream_t)stream);
  } else {
    st = tc.big ? launch_rs<TileBigDirect>(p, (hipStream_t)stream) : launch_rs<TileSmall>(p, (hipStream_t)stream);
  }
  if (st != DITRON_OK) return st;

  ReduceParams r{};
  const size_t slot_bytes = (size_t)m_r * n * 2;
  for (int s = 0; s < world; ++s) {
    if (s == rank) {
      r.slot[s] = fuse ? (const char*)scatter_buf + (size_t)rank * slot_bytes : (const char*)gemm_out + (size_t)rank * slot_bytes;
      r.gate[s] = p.seg_flags + rank;   // the GEMM's flag for the own segment gates every chunk
      r.gate_stride[s] = 0;
    } else {
      r.slot[s] = (const char*)scatter_buf + (size_t)s * slot_bytes;
      // flags preset: the peers' blocks are resident, only the GEMM's own segment gates the sum
      r.gate[s] = mode == Mode::kPreset ? nullptr : p.arr_flags + (size_t)s * chunks_per_slot;
      r.gate_stride[s] = 1;
    }
  }
  r.out = (__bf16*)out;
  r.status = status;
  r.vec_per_chunk = (size_t)(m_r / chunks_per_slot) * n / 8;
  r.chunks = chunks_per_slot;
  r.world = world;
  r.epoch = epoch;
  r.spin_limit = tune.spin_limit;
  // with emulated peers (or everything resident) every flag was raised by the launch before this one
  return launch_reduce(r, /*flags_pending=*/mode == Mode::kExternal, (hipStream_t)stream);
}

extern "C" ditron_status_t ditron_gemm_rs(const void* a, const void* b, int b_layout, void* gemm_out,
                                          const void* const* peer_partials, void* scatter_buf, void* out,
                                          int32_t* signals, int32_t* status, int32_t* schedule_out,
                                          const int* arrival_order, int m, int n, int k_local, int world, int rank,
                                          int chunks_per_slot, int32_t epoch, unsigned flags,
                                          const ditron_tuning_t* tuning, void* stream) {
  return gemm_rs_impl(a, b, b_layout, gemm_out, nullptr, peer_partials, scatter_buf, out, signals, status, schedule_out,
                      arrival_order, m, n, k_local, world, rank, chunks_per_slot, epoch, flags, tuning, stream);
}

extern "C" ditron_status_t ditron_gemm_rs_fuse_scatter(const void* a, const void* b, int b_layout,
                                                       void* const* scatter_dsts, const void* const* peer_partials,
                                                       void* out, int32_t* signals, int32_t* status,
                                                       int32_t* schedule_out, const int* arrival_order, int m, int n,
                                                       int k_local, int world, int rank, int chunks_per_slot,
                                                       int32_t epoch, unsigned flags,
                                                       const ditron_tuning_t* tuning, void* stream) {
  if (!scatter_dsts || world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  return gemm_rs_impl(a, b, b_layout, nullptr, scatter_dsts, peer_partials, scatter_dsts[rank], out, signals, status,
                      schedule_out, arrival_order, m, n, k_local, world, rank, chunks_per_slot, epoch, flags, tuning,
                      stream);
}
