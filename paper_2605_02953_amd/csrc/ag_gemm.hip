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
  const float* a_scales;
  const float* b_scales;
  int32_t* flags;      // [world]
  int32_t* arrivals;   // [world] producer arrival counters
  int32_t* status;
  int32_t* schedule;   // or null
  int m_per_rank, m, n, k, world, rank, nnodes;
  int32_t epoch;
  int num_producers, teams;
  unsigned spin_limit;
  int group_m, num_xcd, per_xcd, npm, npn;
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
  const int pid = xcd_remap(wg, p.npm * p.npn, p.num_xcd, p.per_xcd);
  int pid_m, pid_n;
  grouped_order(pid, p.npm, p.npn, p.group_m, pid_m, pid_n);
  // start on the rows of the rank's own shard, then follow the ring (across nodes: own node first)
  pid_m = p.nnodes > 1 ? tile_row_across_nodes(pid_m, p.m, p.rank, p.world, p.nnodes, T::BM, kOrderGather)
                       : (pid_m + cdiv(p.m_per_rank * p.rank, T::BM)) % p.npm;
  const int m0 = pid_m * T::BM, n0 = pid_n * T::BN;
  const int rank_beg = m0 / p.m_per_rank;
  const int rank_end = (min(m0 + T::BM, p.m) - 1) / p.m_per_rank;
  if (p.schedule && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * (size_t)wg;
    rec[0] = pid_m; rec[1] = pid_n; rec[2] = rank_beg; rec[3] = rank_end;
  }
  flag_wait_block(p.flags, rank_beg, rank_end - rank_beg + 1, p.epoch, p.spin_limit, p.status);

  const uint32_t row_bytes = (uint32_t)p.k * 2u;
  const int M = p.m, N = p.n;
  auto a_row = [=](int r) { return (uint32_t)min(m0 + r, M - 1) * row_bytes; };
  f32x16_t acc[T::NI][T::MI];
  if constexpr (T::B_KN) {
    gemm_mainloop<T>(acc, p.workspace, a_row, p.b, BColumns{(uint32_t)N * 2u, n0, N}, p.k, lds);
  } else {
    auto b_row = [=](int r) { return (uint32_t)min(n0 + r, N - 1) * row_bytes; };
    gemm_mainloop<T>(acc, p.workspace, a_row, p.b, b_row, p.k, lds);
  }
  store_tile_bf16<T>(acc, p.c, (size_t)p.n, m0, n0, M, N, lds);
}

template <class T>
static ditron_status_t launch_ag(AgGemmParams& p, hipStream_t stream) {
  p.npm = cdiv(p.m, T::BM);
  p.npn = cdiv(p.n, T::BN);
  auto kern = ag_gemm_kernel<T>;
  if (!set_dynamic_lds((const void*)kern, T::LDS_BYTES)) return DITRON_ERR_HIP;
  const unsigned grid = (unsigned)(p.num_producers + p.npm * p.npn);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

}  // namespace ditron

using namespace ditron;

extern "C" ditron_status_t ditron_ag_gemm(const void* const* a_shards, const void* b, int b_layout, void* c,
                                          const float* a_scales, const float* b_scales, void* workspace,
                                          int32_t* signals, int32_t* status, int32_t* schedule_out,
                                          const int* arrival_order, int m_per_rank, int n, int k, int world,
                                          int rank, int dtype, int32_t epoch, unsigned flags, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (m_per_rank <= 0 || n <= 0 || k <= 0) return DITRON_ERR_INVALID_ARG;
  if (world % g_num_nodes != 0) return DITRON_ERR_INVALID_ARG;
  if (!b || !c || !workspace || !signals || !status) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(b) || !aligned16(c) || !aligned16(workspace) || !aligned16(signals)) return DITRON_ERR_INVALID_ARG;
  const bool emulate = (flags & DITRON_EMULATE_PRODUCER) != 0;
  const bool external = (flags & DITRON_EXTERNAL_PRODUCER) != 0;
  if (emulate == external) return DITRON_ERR_INVALID_ARG;
  if ((flags & DITRON_DUMP_SCHEDULE) && !schedule_out) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (dtype != DITRON_BF16 && dtype != DITRON_FP8_E4M3) return DITRON_ERR_INVALID_ARG;
  if (emulate) {
    if (!a_shards) return DITRON_ERR_INVALID_ARG;
    for (int s = 0; s < world; ++s)
      if (!a_shards[s] || !aligned16(a_shards[s])) return DITRON_ERR_INVALID_ARG;
    if (arrival_order && !is_permutation(arrival_order, world)) return DITRON_ERR_INVALID_ARG;
  }
  if (dtype == DITRON_FP8_E4M3 || (b_layout == DITRON_B_NK && bf16_ag_is_decode_shaped(m_per_rank * world, n)))
    return ditron_ag_gemm_decode(a_shards, b, b_layout, c, a_scales, b_scales, workspace, signals, status, schedule_out,
                                 arrival_order, m_per_rank, n, k, world, rank, dtype, epoch, flags, stream);
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
  p.a_scales = nullptr;
  p.b_scales = nullptr;
  p.flags = signals;
  p.arrivals = signals + world;
  p.status = status;
  p.schedule = (flags & DITRON_DUMP_SCHEDULE) ? schedule_out : nullptr;
  p.m_per_rank = m_per_rank;
  p.m = m_per_rank * world;
  p.n = n;
  p.k = k;
  p.world = world;
  p.rank = rank;
  p.nnodes = g_num_nodes;
  p.epoch = epoch;
  p.spin_limit = g_spin_limit;
  TileChoice tc = choose_tile(p.m, n, k);
  if (p.nnodes > 1 && !node_order_is_bijection(p.m, tc.block_m, world, p.nnodes, rank, kOrderGather))
    return DITRON_ERR_UNSUPPORTED;
  p.group_m = tc.group_m;
  p.num_xcd = tc.num_xcd;
  p.per_xcd = tc.per_xcd;
  const ProducerPlan pl = plan_producers((size_t)p.m * k * 2, world);
  p.num_producers = emulate ? pl.producers : 0;
  p.teams = pl.teams;
  if (b_layout == DITRON_B_KN) {
    if (tc.big) return launch_ag<TileBigKN>(p, (hipStream_t)stream);
    return launch_ag<TileSmallKN>(p, (hipStream_t)stream);
  }
  if (tc.big && use_direct_staging(k)) return launch_ag<TileBigDirect>(p, (hipStream_t)stream);
  if (tc.big) return launch_ag<TileBig>(p, (hipStream_t)stream);
  return launch_ag<TileSmall>(p, (hipStream_t)stream);
}
