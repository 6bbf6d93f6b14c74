// AllGather-GEMM, one rank's share (paper, Appendix "AllGather GEMM").
//
// One launch holds both roles.  The first `num_producers` work-groups are the emulated
// peers: shard by shard, in delivery order, they copy shard s into rows
// [s*m_per_rank, (s+1)*m_per_rank) of the workspace and then raise flag s (the copy is
// fused into the kernel rather than issued as separate memcpy calls).  Every other
// work-group is one output tile of the consumer GEMM: it maps its index to a tile through
// the chiplet remap, the grouped order and the rank rotation, waits for the flags of the
// shards its rows touch, and only then reads the workspace.  Producer work-groups have the
// lowest indices, so they are dispatched before any consumer can occupy a compute unit.
#include "gemm_core.h"
#include "launch.h"

namespace ditron {

struct AgGemmParams {
  const void* shard[DITRON_MAX_WORLD];
  int order[DITRON_MAX_WORLD];
  char* workspace;
  const char* b;
  __bf16* c;
  int32_t* flags;      // [world]
  int32_t* arrivals;   // [world] producer arrival counters
  int32_t* status;
  int32_t* schedule;   // or null
  int timing;          // schedule records hold time stamps instead
  int m_per_rank, m, n, k, world, rank, nnodes;
  int32_t epoch;
  int num_producers, teams;
  unsigned spin_limit;
  int wait;            // 0: every shard is resident, the flags are not looked at
  TileOrder tiling;
};

template <class T>
__global__ __launch_bounds__(T::THREADS) void ag_gemm_kernel(const AgGemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  if ((int)blockIdx.x < p.num_producers) {
    const size_t shard_bytes = (size_t)p.m_per_rank * p.k * 2;
    produce_chunks<T::THREADS>(
        p.world, shard_bytes, blockIdx.x, p.num_producers, p.teams, p.epoch,
        [&](int i) { return (void*)(p.workspace + (size_t)p.order[i] * shard_bytes); },
        [&](int i) { return p.shard[p.order[i]]; }, [&](int i) { return p.flags + p.order[i]; },
        [&](int i) { return p.arrivals + p.order[i]; });
    return;
  }
  const int wg = blockIdx.x - p.num_producers;
  const TileSpan t = tile_of_workgroup(wg, p.tiling, kOrderGather, p.m, p.m_per_rank, p.rank, p.world, p.nnodes, T::BM);
  const int m0 = t.pid_m * T::BM, n0 = t.pid_n * T::BN;
  const unsigned long long ts_start = p.timing ? wall_clock64() : 0;
  if (p.schedule && !p.timing && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * (size_t)wg;
    rec[0] = t.pid_m; rec[1] = t.pid_n; rec[2] = t.first; rec[3] = t.last;
  }
  if (p.wait) flag_wait_block(p.flags, t.first, t.last - t.first + 1, p.epoch, p.spin_limit, p.status);
  const unsigned long long ts_ready = p.timing ? wall_clock64() : 0;

  const uint32_t row_bytes = (uint32_t)p.k * 2u;
  const int M = p.m, N = p.n;
  auto a_row = [=](int r) { return (uint32_t)min(m0 + r, M - 1) * row_bytes; };
  typename T::Acc acc;
  if constexpr (T::B_KN) {
    gemm_mainloop<T>(acc, p.workspace, a_row, p.b, BColumns{(uint32_t)N * 2u, n0, N}, p.k, lds);
  } else {
    auto b_row = [=](int r) { return (uint32_t)min(n0 + r, N - 1) * row_bytes; };
    gemm_mainloop<T>(acc, p.workspace, a_row, p.b, b_row, p.k, lds);
  }
  store_tile_bf16<T>(acc, p.c, (size_t)p.n, m0, n0, M, N, lds);
  if (p.timing && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * (size_t)wg;
    rec[0] = (int32_t)(ts_start & 0x7fffffff); rec[1] = rec[0];
    rec[2] = (int32_t)(ts_ready & 0x7fffffff); rec[3] = (int32_t)(wall_clock64() & 0x7fffffff);
  }
}

template <class T>
static ditron_status_t launch_ag(AgGemmParams& p, hipStream_t stream) {
  p.tiling.npm = cdiv(p.m, T::BM);
  p.tiling.npn = cdiv(p.n, T::BN);
  if (!set_dynamic_lds<ag_gemm_kernel<T>>(T::LDS_BYTES)) return DITRON_ERR_HIP;
  const unsigned grid = (unsigned)(p.num_producers + p.tiling.npm * p.tiling.npn);
  hipLaunchKernelGGL(ag_gemm_kernel<T>, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

}  // namespace ditron

using namespace ditron;

extern "C" ditron_status_t ditron_ag_gemm(const void* const* a_shards, const void* b, int b_layout, void* c,
                                          const float* a_scales, const float* b_scales, void* workspace,
                                          int32_t* signals, int32_t* status, int32_t* schedule_out,
                                          const int* arrival_order, int m_per_rank, int n, int k, int world,
                                          int rank, int dtype, int32_t epoch, unsigned flags,
                                          const ditron_tuning_t* tuning, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (m_per_rank <= 0 || n <= 0 || k <= 0) return DITRON_ERR_INVALID_ARG;
  const Tuning tune = resolve_tuning(tuning, world);
  if (!tune.valid) return DITRON_ERR_INVALID_ARG;
  if (!b || !c || !workspace || !signals || !status) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(b) || !aligned16(c) || !aligned16(workspace) || !aligned16(signals)) return DITRON_ERR_INVALID_ARG;
  const Mode mode = producer_mode(flags);
  if (mode == Mode::kInvalid) return DITRON_ERR_INVALID_ARG;
  const bool emulate = mode == Mode::kEmulate;
  if ((flags & (DITRON_DUMP_SCHEDULE | DITRON_DUMP_TIMING)) && !schedule_out) return DITRON_ERR_INVALID_ARG;
  if ((flags & DITRON_DUMP_SCHEDULE) && (flags & DITRON_DUMP_TIMING)) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (dtype != DITRON_BF16 && dtype != DITRON_FP8_E4M3) return DITRON_ERR_INVALID_ARG;
  if (emulate) {
    if (!a_shards) return DITRON_ERR_INVALID_ARG;
    for (int s = 0; s < world; ++s)
      if (!a_shards[s] || !aligned16(a_shards[s])) return DITRON_ERR_INVALID_ARG;
    if (arrival_order && !is_permutation(arrival_order, world)) return DITRON_ERR_INVALID_ARG;
  }
  const bool decode_shaped = dtype == DITRON_FP8_E4M3 || (b_layout == DITRON_B_NK && bf16_ag_is_decode_shaped(m_per_rank * world, n));
  if ((flags & DITRON_EPOCH_IN_MEMORY) && !decode_shaped) return DITRON_ERR_UNSUPPORTED;
  if (decode_shaped)
    return ditron_ag_gemm_decode(a_shards, b, b_layout, c, a_scales, b_scales, workspace, signals, status, schedule_out,
                                 arrival_order, m_per_rank, n, k, world, rank, dtype, epoch, flags, tuning, stream);
  if (k % 8 != 0 || n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit((size_t)m_per_rank * world, k, 2) || !fits_32bit(n, k, 2)) return DITRON_ERR_UNSUPPORTED;

  AgGemmParams p{};
  for (int i = 0; i < world; ++i) {
    p.shard[i] = emulate ? a_shards[i] : nullptr;
    p.order[i] = arrival_order ? arrival_order[i] : (rank + i) % world;
  }
  p.workspace = (char*)workspace;
  p.b = (const char*)b;
  p.c = (__bf16*)c;
  p.flags = signals;
  p.arrivals = signals + world;
  p.status = status;
  p.schedule = (flags & (DITRON_DUMP_SCHEDULE | DITRON_DUMP_TIMING)) ? schedule_out : nullptr;
  p.timing = (flags & DITRON_DUMP_TIMING) != 0;
  p.m_per_rank = m_per_rank;
  p.m = m_per_rank * world;
  p.n = n;
  p.k = k;
  p.world = world;
  p.rank = rank;
  p.nnodes = tune.num_nodes;
  p.epoch = epoch;
  p.spin_limit = tune.spin_limit;
  p.wait = mode != Mode::kPreset;
  TileChoice tc = choose_tile(p.m, n, k, b_layout == DITRON_B_NK);
  if (p.nnodes > 1 && !node_order_is_bijection(p.m, tc.block_m, world, p.nnodes, rank, kOrderGather))
    return DITRON_ERR_UNSUPPORTED;
  p.tiling.group_m = tc.group_m;
  p.tiling.num_xcd = tc.num_xcd;
  p.tiling.per_xcd = tc.per_xcd;
  const ProducerPlan pl = plan_producers((size_t)p.m * k * 2, world);
  p.num_producers = emulate ? pl.producers : 0;
  p.teams = pl.teams;
  if (b_layout == DITRON_B_KN) {
    if (tc.big) return launch_ag<TileBigKN>(p, (hipStream_t)stream);
    return launch_ag<TileSmallKN>(p, (hipStream_t)stream);
  }
  if (tc.big) {
    if (tc.block_n == 224) return launch_ag<TileBigDirect224>(p, (hipStream_t)stream);
    if (tc.block_n == 192) return launch_ag<TileBigDirect192>(p, (hipStream_t)stream);
    return launch_ag<TileBigDirect>(p, (hipStream_t)stream);
  }
  return launch_ag<TileSmall>(p, (hipStream_t)stream);
}
