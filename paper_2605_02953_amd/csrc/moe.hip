// MoE AllGather + grouped GEMM, one rank's share (paper: "ag_group_gemm" of the kernel
// list; tile ordering after `threadblock_swizzle_ag_moe_kernel`, Appendix "Swizzle").
//
// Launch 1.  The first work-groups (integer only, up to eight sharing the scan plus one for the
// schedule): per-(rank, expert) histogram, exclusive scan of the local experts' totals, stable
// gather index, then the tile list: every local expert's rows are cut into BLOCK_M row tiles, each
// tile learns the span of source ranks its rows come from and the ring stage at which the last of
// them arrives, and tiles are emitted grouped by expert, ascending stage, ties in original order.
// The other work-groups are the emulated peers: they copy the token shards into the workspace in
// delivery order and raise one flag per shard.  The all-gather does not depend on the routing, so
// it starts with the call and runs beside the routing work-groups (which leave the rest of the chip idle).
// Launch 2: every work-group takes one (tile, column block), waits for the shard flags of its
// tile, gathers its rows through gather_idx while staging them in LDS and multiplies by its
// expert's weights.
#include "gemm_core.h"
#include "launch.h"

namespace ditron {

constexpr int kRouteThreads = 1024;
constexpr int kRouteWaves = kRouteThreads / 64;
constexpr int kMaxExperts = 256;       // experts (global) the routing kernel can histogram
constexpr int kMaxLocalExperts = 64;
constexpr int kMaxTilesLds = 4096;     // tile stages kept in LDS by the schedule step
constexpr int kRouteGroupsMax = 8;     // work-groups that share the routing scan
// what a routing work-group hands to the others: its (rank, expert) histogram, its totals of the local
// experts, and the smallest flat index at which it met an id that names no expert
constexpr int kPartLocal = DITRON_MAX_WORLD * kMaxExperts;
constexpr int kPartBad = kPartLocal + kMaxLocalExperts;
constexpr int kRoutePartWords = kPartBad + 64;
static_assert(kRouteGroupsMax * kRoutePartWords * 4 == DITRON_MOE_ROUTE_SCRATCH_BYTES, "scratch size declared at the boundary");
constexpr int kNoBadId = 0x7fffffff;
constexpr int kWalkExperts = 16;       // up to this many local experts a work-group finds its expert by a scalar walk

struct MoeRouteParams {
  const int32_t* topk_ids;   // [tokens * top_k]
  int32_t* counts;           // [world * num_experts]
  int32_t* expert_offsets;   // [num_local + 1]
  int32_t* gather_idx;       // [max_rows]
  int32_t* tile_records;     // [0] = ntiles ; 4 words per tile ; then max_tiles words: first row of the tile
  int32_t* status;
  int tokens_per_rank, top_k, num_experts, expert_begin, num_local, max_rows, max_tiles;
  int world, rank, block_m;
  // routing work-groups 0 .. groups-1 and the scheduling work-group `groups`
  int groups;
  int32_t* route_flags;      // [groups]
  int32_t* parts;            // [groups][kRoutePartWords]
  unsigned spin_limit;
  // the emulated peers (work-groups groups+1 .. groups+num_producers)
  const void* shard[DITRON_MAX_WORLD];
  int order[DITRON_MAX_WORLD];
  char* workspace;
  int32_t* flags;
  int32_t* arrivals;
  size_t shard_bytes;
  int32_t epoch;
  int num_producers, teams;
};

// Work-groups 0 .. G-1 share the scan of the assignments: each owns one contiguous range, cut into one
// contiguous range per wave, so that positions inside an expert follow the flat assignment index whatever G
// is.  A work-group histograms its range, hands its partial tables to the others through memory (one flag
// per work-group, bounded wait), and then places its own assignments: the first output position of (work-
// group, wave, expert) is the expert's offset plus what the ranges before it hold of that expert.
// Work-group G sums the histograms and writes counts, offsets and the tile list.  All G + 1 have the lowest
// indices of the launch, so they are resident before anything else and the waits end.
__global__ __launch_bounds__(kRouteThreads) void moe_route_kernel(const MoeRouteParams p) {
  __shared__ int s_counts[DITRON_MAX_WORLD * kMaxExperts];       // [world][num_experts]
  __shared__ int s_offsets[kMaxLocalExperts + 1];
  __shared__ int s_wave_base[kRouteWaves][kMaxLocalExperts];     // running output position per (wave, expert)
  __shared__ int s_tile_acc[kMaxLocalExperts + 1];               // exclusive prefix of tiles per expert
  __shared__ int s_cum[kMaxLocalExperts][DITRON_MAX_WORLD];      // inclusive per-rank cumulative rows per expert
  __shared__ int s_total[kMaxLocalExperts], s_before[kMaxLocalExperts];
  __shared__ int s_stage[kMaxTilesLds];
  __shared__ int s_bad;                                          // smallest flat index holding an id outside [0, E)
  const int G = p.groups;
  if ((int)blockIdx.x > G) {
    // streaming stores: the grouped GEMM that reads the workspace is a later launch
    produce_chunks<kRouteThreads, true>(
        p.world, p.shard_bytes, blockIdx.x - G - 1, p.num_producers, p.teams, p.epoch,
        [&](int i) { return (void*)(p.workspace + (size_t)p.order[i] * p.shard_bytes); },
        [&](int i) { return p.shard[p.order[i]]; }, [&](int i) { return p.flags + p.order[i]; },
        [&](int i) { return p.arrivals + p.order[i]; });
    return;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int F = p.world * p.tokens_per_rank * p.top_k;
  const int per_shard = p.tokens_per_rank * p.top_k;
  const int E = p.num_experts, EL = p.num_local, WE = p.world * E;

  if ((int)blockIdx.x == G) {
    // ---------------------------------------------------------------- counts, offsets, tile list
    flag_wait_block(p.route_flags, 0, G, p.epoch, p.spin_limit, p.status);
    for (int i = tid; i < WE; i += kRouteThreads) {
      int c = 0;
      for (int g = 0; g < G; ++g) c += p.parts[g * kRoutePartWords + i];
      s_counts[i] = c;
      p.counts[i] = c;
    }
    if (tid == 0) {
      int bad = kNoBadId;
      for (int g = 0; g < G; ++g) bad = min(bad, p.parts[g * kRoutePartWords + kPartBad]);
      s_bad = bad;
    }
    __syncthreads();
    if (s_bad != kNoBadId) {
      // an id that names no expert: reported, never dropped silently (the counts would no longer sum to
      // tokens * top_k); no tile is scheduled
      if (tid == 0) {
        p.status[0] = DITRON_ERR_INVALID_ARG;
        p.status[1] = s_bad;
        p.tile_records[0] = 0;
      }
      return;
    }
    // per-rank cumulative rows of the local experts; exclusive scan of their totals
    if (tid < EL) {
      int run = 0;
      for (int s = 0; s < p.world; ++s) {
        run += s_counts[s * E + p.expert_begin + tid];
        s_cum[tid][s] = run;
      }
    }
    __syncthreads();
    if (tid == 0) {
      int run = 0, tiles = 0;
      for (int j = 0; j < EL; ++j) {
        s_offsets[j] = run;
        s_tile_acc[j] = tiles;
        const int n_j = s_cum[j][p.world - 1];
        run += n_j;
        tiles += cdiv(n_j, p.block_m);
      }
      s_offsets[EL] = run;
      s_tile_acc[EL] = tiles;
    }
    __syncthreads();
    for (int j = tid; j <= EL; j += kRouteThreads) p.expert_offsets[j] = s_offsets[j];
    const int R = s_offsets[EL];
    const int ntiles = s_tile_acc[EL];
    if (R > p.max_rows || ntiles > p.max_tiles || ntiles > kMaxTilesLds) {
      if (tid == 0) {
        p.status[0] = DITRON_ERR_WORKSPACE;
        p.status[2] = R;
        p.tile_records[0] = 0;
      }
      return;
    }
    // stage of a tile: position in the ring order rank, rank+1, ... of the last source rank among its rows
    for (int t = tid; t < ntiles; t += kRouteThreads) {
      int j = 0;
      while (s_tile_acc[j + 1] <= t) ++j;
      const int q0 = (t - s_tile_acc[j]) * p.block_m;
      const int q1 = min(q0 + p.block_m, s_cum[j][p.world - 1]);
      int seg_start = 0, seg_end = 0;
      for (int s = 0; s < p.world; ++s) {
        seg_start += (s_cum[j][s] <= q0);
        seg_end += (s_cum[j][s] <= q1 - 1);
      }
      int stage = 0;
      for (int s = seg_start; s <= seg_end; ++s) stage = max(stage, (s - p.rank + p.world) % p.world);
      s_stage[t] = stage | (seg_start << 8) | (seg_end << 16);
    }
    __syncthreads();
    int32_t* rec = p.tile_records + 1;
    int32_t* row0 = p.tile_records + 1 + 4 * p.max_tiles;
    for (int t = tid; t < ntiles; t += kRouteThreads) {
      int j = 0;
      while (s_tile_acc[j + 1] <= t) ++j;
      const int mine = s_stage[t] & 0xFF;
      int before = 0;
      for (int u = s_tile_acc[j]; u < s_tile_acc[j + 1]; ++u) {
        const int other = s_stage[u] & 0xFF;
        before += (other < mine) || (other == mine && u < t);
      }
      const int pos = s_tile_acc[j] + before;
      rec[4 * pos + 0] = j;
      rec[4 * pos + 1] = t;
      rec[4 * pos + 2] = (s_stage[t] >> 8) & 0xFF;
      rec[4 * pos + 3] = (s_stage[t] >> 16) & 0xFF;
      row0[pos] = s_offsets[j] + (t - s_tile_acc[j]) * p.block_m;
    }
    if (tid == 0) p.tile_records[0] = ntiles;
    return;
  }

  // ------------------------------------------------------------------ routing work-group g
  const int g = blockIdx.x;
  for (int i = tid; i < WE; i += kRouteThreads) s_counts[i] = 0;
  for (int i = tid; i < kRouteWaves * kMaxLocalExperts; i += kRouteThreads) (&s_wave_base[0][0])[i] = 0;
  if (tid == 0) s_bad = kNoBadId;
  __syncthreads();

  // histogram over (source rank, expert), and per-wave totals for the local experts.  The ids are fetched
  // kBatch steps at a time so that the loads overlap instead of queueing one by one.
  constexpr int kBatch = 16;
  const int per_wave = cdiv(cdiv(F, G * kRouteWaves), 64) * 64;
  const int w_begin = (int)min((long)(g * kRouteWaves + wave) * per_wave, (long)F), w_end = min(w_begin + per_wave, F);
  for (int f0 = w_begin; f0 < w_end; f0 += 64 * kBatch) {
    int e[kBatch];
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int f = f0 + b * 64 + lane;
      e[b] = f < w_end ? p.topk_ids[f] : -1;
    }
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int f = f0 + b * 64 + lane;
      if (f >= w_end) continue;
      if (e[b] >= 0 && e[b] < E) {
        atomicAdd(&s_counts[(f / per_shard) * E + e[b]], 1);
        const int j = e[b] - p.expert_begin;
        if (j >= 0 && j < EL) atomicAdd(&s_wave_base[wave][j], 1);
      } else {
        atomicMin(&s_bad, f);
      }
    }
  }
  __syncthreads();
  int32_t* part = p.parts + g * kRoutePartWords;
  for (int i = tid; i < WE; i += kRouteThreads) part[i] = s_counts[i];
  if (tid < EL) {
    int c = 0;
    for (int w = 0; w < kRouteWaves; ++w) c += s_wave_base[w][tid];
    part[kPartLocal + tid] = c;
  }
  if (tid == 0) part[kPartBad] = s_bad;
  __syncthreads();
  if (tid == 0) flag_raise(p.route_flags + g, p.epoch);
  flag_wait_block(p.route_flags, 0, G, p.epoch, p.spin_limit, p.status);

  // every routing work-group takes the same decisions from the same tables
  if (tid < EL) {
    int total = 0, before = 0;
    for (int h = 0; h < G; ++h) {
      const int c = p.parts[h * kRoutePartWords + kPartLocal + tid];
      total += c;
      before += h < g ? c : 0;
    }
    s_total[tid] = total;
    s_before[tid] = before;
  }
  if (tid == 64) {
    int bad = kNoBadId;
    for (int h = 0; h < G; ++h) bad = min(bad, p.parts[h * kRoutePartWords + kPartBad]);
    s_bad = bad;
  }
  __syncthreads();
  if (s_bad != kNoBadId) return;
  if (tid == 0) {
    int run = 0, tiles = 0;
    for (int j = 0; j < EL; ++j) {
      s_offsets[j] = run;
      run += s_total[j];
      tiles += cdiv(s_total[j], p.block_m);
    }
    s_offsets[EL] = run;
    s_tile_acc[EL] = tiles;
  }
  __syncthreads();
  if (s_offsets[EL] > p.max_rows || s_tile_acc[EL] > p.max_tiles || s_tile_acc[EL] > kMaxTilesLds) return;

  // first output position of every (wave, expert) of this work-group
  if (tid < EL) {
    int run = s_offsets[tid] + s_before[tid];
    for (int w = 0; w < kRouteWaves; ++w) {
      const int c = s_wave_base[w][tid];
      s_wave_base[w][tid] = run;
      run += c;
    }
  }
  __syncthreads();

  // stable placement: 64 assignments at a time.  The lanes that hold the same local expert find
  // each other with one ballot per bit of the expert index (a lane keeps the lanes that agree with
  // it on every bit) and rank themselves by counting the lanes below them.  The first lane of each
  // group moves the wave's running output position of that expert past the group with one LDS atomic,
  // whose return value is the group's first position; the others receive it by a lane shuffle.  The
  // row of running positions is private to the wave and a wave's LDS atomics execute in order, so
  // consecutive rounds see each other's advances.  The cost per round does not grow with the number
  // of local experts beyond the number of index bits.
  const int nbits = EL > 1 ? 32 - __builtin_clz(EL - 1) : 0;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int fb = w_begin; fb < w_end; fb += 64 * kBatch) {
    int jj[kBatch];
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int f = fb + b * 64 + lane;
      int j = -1;
      if (f < w_end) {
        j = p.topk_ids[f] - p.expert_begin;
        if (j < 0 || j >= EL) j = -1;
      }
      jj[b] = j;
    }
#pragma unroll
    for (int b = 0; b < kBatch; ++b) {
      const int f = fb + b * 64 + lane;
      const int j = jj[b];
      const bool local = j >= 0;
      unsigned long long same = __ballot(local);
      if (same == 0) continue;
      for (int bit = 0; bit < nbits; ++bit) {
        const bool set = local && ((j >> bit) & 1);
        const unsigned long long m = __ballot(set);
        same &= set ? m : ~m;
      }
      const int rank = __popcll(same & below), count = __popcll(same);
      int base = 0;
      if (local && rank == 0) base = atomicAdd(&s_wave_base[wave][j], count);
      base = __shfl(base, local ? __ffsll((long long)same) - 1 : lane);
      // (the range test only matters after a timed-out wait, when the tables may be incomplete)
      if (local && (unsigned)(base + rank) < (unsigned)p.max_rows) p.gather_idx[base + rank] = f;
    }
  }
}

struct MoeGemmParams {
  const char* workspace;
  const char* w;
  __bf16* y;
  const int32_t* expert_offsets;
  const int32_t* gather_idx;
  const int32_t* tile_records;
  const int32_t* flags;
  int32_t* status;
  int tokens_per_rank, hidden, inter, top_k, world, max_tiles, npn, num_local, num_xcd;   // hidden: contraction length, inter: output width
  int rows_in_place;   // 1: row p of the left operand is row p of `workspace` (already grouped by expert), no gather
  int32_t* inverse_idx;   // if set: the work-groups of column block 0 also write inverse_idx[gather_idx[p]] = p for their rows
  int assignments;
  int32_t epoch;
  unsigned spin_limit;
  int wait;   // 0: the token shards are resident, the flags are not looked at
};

// NST > 0: operands through a ring of NST LDS stages filled by four extra waves (expert weights stream from
// HBM: see gemm_mainloop_ring_split)
// WALK: the launch has fewer work-groups than items and every work-group walks down its chiplet's run with the
// stride of the grid (short tiles: a work-group start costs as much as the tile).
template <class T, int NST = 0, bool WALK = false>
__global__ __launch_bounds__(NST > 0 ? 2 * T::THREADS : T::THREADS) void moe_grouped_gemm_kernel(const MoeGemmParams p) {
  static_assert(!WALK || NST == 0, "the loading waves of the ring leave the kernel after one item");
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // Work-group -> (row tile, column block).  All (row tile, column block) items are put in one list, expert
  // after expert, inside an expert column block after column block, the expert's row tiles (one to three) of
  // a column block next to each other; the list is cut into as many equal runs as there are chiplets and
  // chiplet x (the work-groups with index = x mod 8) takes run x.  Neighbours in the list share a block of the
  // expert's weights (same column block) or the gathered rows (same row tile), so each comes from memory about
  // once, and every chiplet has the same number of tiles (an expert per chiplet moves as few bytes but leaves
  // the chiplets of small experts idle while the large ones run two rounds).  The row tiles of expert j are
  // the positions [first_j, first_j + ceil(n_j / BLOCK_M)) of the tile list, in arrival-stage order.
  const int wg = blockIdx.x;
  const int ntiles = p.tile_records[0];
  if (ntiles <= 0) return;   // nothing routed here, or the routing launch reported an error
  const int per_xcd = cdiv(ntiles * p.npn, p.num_xcd);
  const int slots_in_grid = WALK ? gridDim.x / p.num_xcd : per_xcd;
  // lane j of every wave: the row tiles of expert j and of the experts before it (at most 64 local experts)
  const int lane_j = threadIdx.x & 63;
  int nt_j = 0, before_j = 0;
  if (WALK || p.num_local > kWalkExperts) {
    nt_j = lane_j < p.num_local ? cdiv(p.expert_offsets[lane_j + 1] - p.expert_offsets[lane_j], T::BM) : 0;
    before_j = nt_j;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int v = __shfl_up(before_j, d);
      if (lane_j >= d) before_j += v;
    }
    before_j -= nt_j;
  }
  for (int slot = wg / p.num_xcd; slot < per_xcd; slot += slots_in_grid) {
  const int item = (wg % p.num_xcd) * per_xcd + slot;
  if (item >= ntiles * p.npn) return;
  int nt, before;
  if (WALK || p.num_local > kWalkExperts) {
    // the expert whose items [before_j npn, (before_j + nt_j) npn) hold this one
    const unsigned long long holds = __ballot(item >= before_j * p.npn && item < (before_j + nt_j) * p.npn);
    if (holds == 0) return;
    const int owner = __ffsll((long long)holds) - 1;
    // (read into scalar registers: the tile's addresses derive from them and must stay wave-uniform)
    nt = __builtin_amdgcn_readlane(nt_j, owner);
    before = __builtin_amdgcn_readlane(before_j, owner);
  } else {
    // a handful of experts: a scalar walk over their offsets
    nt = 0;
    before = 0;
    for (int j = 0; j < p.num_local; ++j) {
      nt = cdiv(p.expert_offsets[j + 1] - p.expert_offsets[j], T::BM);
      if (item < (before + nt) * p.npn) break;
      before += nt;
    }
    if (nt == 0) return;
  }
  const int pid_n = (item - before * p.npn) / nt;
  const int pos = before + (item - before * p.npn) % nt;
  const int32_t* rec = p.tile_records + 1 + 4 * pos;
  const int j = rec[0], seg_start = rec[2], seg_end = rec[3];
  const int p0 = p.tile_records[1 + 4 * p.max_tiles + pos];
  const int p_end = min(p0 + T::BM, p.expert_offsets[j + 1]);
  if (p.wait) flag_wait_block(p.flags, seg_start, seg_end - seg_start + 1, p.epoch, p.spin_limit, p.status);
  if (p.inverse_idx && pid_n == 0) {
    // every row belongs to exactly one row tile, and every row tile has one work-group of column block 0
    for (int row = p0 + (int)threadIdx.x; row < p_end; row += (int)blockDim.x) {
      const int f = p.gather_idx[row];
      if (f >= 0 && f < p.assignments) p.inverse_idx[f] = row;
    }
  }

  const int n0 = pid_n * T::BN;
  const uint32_t row_bytes = (uint32_t)p.hidden * 2u;
  const char* wj = p.w + (size_t)j * p.inter * row_bytes;
  const int32_t* gidx = p.gather_idx;
  const int top_k = p.top_k, N = p.inter;
  // the gather happens here: a tile row is fetched from the token its assignment belongs to
  const int in_place = p.rows_in_place;
  auto a_row = [=](int r) {
    const int row = min(p0 + r, p_end - 1);
    return (uint32_t)(in_place ? row : gidx[row] / top_k) * row_bytes;
  };
  typename T::Acc acc;
  if constexpr (T::B_KN) {   // expert weights stored [hidden, inter]: same bytes per expert, inter contiguous
    gemm_mainloop<T>(acc, p.workspace, a_row, wj, BColumns{(uint32_t)N * 2u, n0, N}, p.hidden, lds);
  } else {
    auto b_row = [=](int r) { return (uint32_t)min(n0 + r, N - 1) * row_bytes; };
    if constexpr (NST > 0) {
      if (!gemm_mainloop_ring_split<T, NST>(acc, p.workspace, a_row, wj, b_row, p.hidden, lds)) {
        __syncthreads();   // the loading waves meet the barrier at the head of the epilogue and leave
        return;
      }
    } else {
      gemm_mainloop<T>(acc, p.workspace, a_row, wj, b_row, p.hidden, lds);
    }
  }
  store_tile_bf16<T>(acc, p.y, (size_t)p.inter, p0, n0, p_end, N, lds);
  if constexpr (!WALK) return;
  __syncthreads();   // the parked tile has been read: the stages are idle for the next item
  }
}

}  // namespace ditron

using namespace ditron;


extern "C" int ditron_moe_max_tiles(int max_rows, int num_local_experts) {
  if (max_rows < 0 || num_local_experts < 0) return 0;
  return cdiv(max_rows, kMoeBlockM) + num_local_experts;
}

template <class T, int NST = 0>
static ditron_status_t launch_moe_gemm(MoeGemmParams& g, int max_tiles, hipStream_t s) {
  g.npn = cdiv(g.inter, T::BN);
  constexpr int kLds = NST > 0 ? NST * T::STAGE_BYTES : T::LDS_BYTES;
  static_assert(kLds <= 160 * 1024, "LDS of one compute unit");
  if (!set_dynamic_lds<moe_grouped_gemm_kernel<T, NST>>(kLds)) return DITRON_ERR_HIP;
  // every chiplet takes an equal share of the (row tile, column block) items
  const unsigned grid = (unsigned)(g.num_xcd * cdiv(max_tiles * g.npn, g.num_xcd));
  hipLaunchKernelGGL((moe_grouped_gemm_kernel<T, NST>), dim3(grid), dim3(NST > 0 ? 2 * T::THREADS : T::THREADS), kLds, s, g);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

// The same with at most `resident` work-groups, which share the items.
template <class T>
static ditron_status_t launch_moe_gemm_walk(MoeGemmParams& g, int max_tiles, int resident, hipStream_t s) {
  g.npn = cdiv(g.inter, T::BN);
  if (!set_dynamic_lds<moe_grouped_gemm_kernel<T, 0, true>>(T::LDS_BYTES)) return DITRON_ERR_HIP;
  const unsigned items = (unsigned)(g.num_xcd * cdiv(max_tiles * g.npn, g.num_xcd));
  const unsigned grid = std::min(items, (unsigned)(g.num_xcd * cdiv(resident, g.num_xcd)));
  hipLaunchKernelGGL((moe_grouped_gemm_kernel<T, 0, true>), dim3(grid), dim3(T::THREADS), T::LDS_BYTES, s, g);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

extern "C" ditron_status_t ditron_moe_ag_grouped_gemm(
    const void* const* x_shards, const int32_t* topk_ids, const void* w, int w_layout, void* y, int32_t* counts,
    int32_t* expert_offsets, int32_t* gather_idx, int32_t* tile_records, void* workspace, int32_t* signals,
    int32_t* status, const int* arrival_order, int tokens_per_rank, int hidden, int inter, int num_experts,
    int top_k, int expert_begin, int num_local_experts, int max_rows, int world, int rank, int32_t epoch,
    unsigned flags, const ditron_tuning_t* tuning, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (tokens_per_rank <= 0 || hidden <= 0 || inter <= 0 || num_experts <= 0 || top_k <= 0 || max_rows <= 0)
    return DITRON_ERR_INVALID_ARG;
  if (expert_begin < 0 || num_local_experts <= 0 || expert_begin + num_local_experts > num_experts)
    return DITRON_ERR_INVALID_ARG;
  if (!topk_ids || !w || !y || !counts || !expert_offsets || !gather_idx || !tile_records || !workspace ||
      !signals || !status)
    return DITRON_ERR_INVALID_ARG;
  if (!aligned16(w) || !aligned16(y) || !aligned16(workspace) || !aligned16(signals)) return DITRON_ERR_INVALID_ARG;
  const Mode mode = producer_mode(flags);
  if (flags & DITRON_EPOCH_IN_MEMORY) return DITRON_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning, 1);
  if (mode == Mode::kInvalid || !tune.valid) return DITRON_ERR_INVALID_ARG;
  const bool emulate = mode == Mode::kEmulate;
  if (w_layout != DITRON_B_KN && w_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (emulate) {
    if (!x_shards) return DITRON_ERR_INVALID_ARG;
    for (int s = 0; s < world; ++s)
      if (!x_shards[s] || !aligned16(x_shards[s])) return DITRON_ERR_INVALID_ARG;
    if (arrival_order && !is_permutation(arrival_order, world)) return DITRON_ERR_INVALID_ARG;
  }
  if (hidden % 8 != 0 || inter % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit((size_t)world * tokens_per_rank, hidden, 2) || !fits_32bit(inter, hidden, 2))
    return DITRON_ERR_UNSUPPORTED;
  if (num_experts > kMaxExperts || num_local_experts > kMaxLocalExperts) return DITRON_ERR_UNSUPPORTED;
  if ((long)world * num_experts > (long)DITRON_MAX_WORLD * kMaxExperts) return DITRON_ERR_UNSUPPORTED;
  const int max_tiles = ditron_moe_max_tiles(max_rows, num_local_experts);
  if (max_tiles > kMaxTilesLds) return DITRON_ERR_UNSUPPORTED;
  if ((long)world * tokens_per_rank * top_k > 0x7fffffffL) return DITRON_ERR_UNSUPPORTED;

  hipStream_t s = (hipStream_t)stream;
  MoeRouteParams r{};
  r.topk_ids = topk_ids;
  r.counts = counts;
  r.expert_offsets = expert_offsets;
  r.gather_idx = gather_idx;
  r.tile_records = tile_records;
  r.status = status;
  r.tokens_per_rank = tokens_per_rank;
  r.top_k = top_k;
  r.num_experts = num_experts;
  r.expert_begin = expert_begin;
  r.num_local = num_local_experts;
  r.max_rows = max_rows;
  r.max_tiles = max_tiles;
  r.world = world;
  r.rank = rank;
  const MoeTile mt = choose_moe_tile(moe_expected_rows((long)world * tokens_per_rank, top_k, num_experts, num_local_experts),
                                     num_local_experts, inter);
  r.block_m = mt.block_m;
  for (int i = 0; i < world; ++i) {
    r.shard[i] = emulate ? x_shards[i] : nullptr;
    r.order[i] = arrival_order ? arrival_order[i] : (rank + i) % world;
  }
  r.workspace = (char*)workspace;
  r.flags = signals;
  r.arrivals = signals + world;
  // one routing work-group per 4096 assignments (three or four rounds of 64 per wave), eight at most
  const long assignments = (long)world * tokens_per_rank * top_k;
  r.groups = tune.moe_route_groups ? tune.moe_route_groups : (int)std::min<long>(kRouteGroupsMax, std::max<long>(1, assignments / 4096));
  r.route_flags = signals + 4 * world;   // behind the flags and counters of a one-chunk layout
  r.parts = (int32_t*)((char*)workspace + align256((size_t)world * tokens_per_rank * hidden * 2));
  r.spin_limit = tune.spin_limit;
  r.shard_bytes = (size_t)tokens_per_rank * hidden * 2;
  r.epoch = epoch;
  // as many work-groups (of 1024 threads here) as the plan for 256-thread producers: measured best of
  // a quarter, half, the same and twice as many (159, 127, 105, 125 us for the whole cfg 4 step)
  const ProducerPlan pl = plan_producers((size_t)world * r.shard_bytes, world);
  r.num_producers = emulate ? pl.producers : 0;
  r.teams = std::min(pl.teams, std::max(1, r.num_producers));
  hipLaunchKernelGGL(moe_route_kernel, dim3(r.groups + 1 + r.num_producers), dim3(kRouteThreads), 0, s, r);
  if (hipGetLastError() != hipSuccess) return DITRON_ERR_HIP;

  MoeGemmParams g{};
  g.workspace = (const char*)workspace;
  g.w = (const char*)w;
  g.y = (__bf16*)y;
  g.expert_offsets = expert_offsets;
  g.gather_idx = gather_idx;
  g.tile_records = tile_records;
  g.flags = signals;
  g.status = status;
  g.tokens_per_rank = tokens_per_rank;
  g.hidden = hidden;
  g.inter = inter;
  g.top_k = top_k;
  g.world = world;
  g.max_tiles = max_tiles;
  g.num_local = num_local_experts;
  g.num_xcd = 8;
  g.epoch = epoch;
  g.spin_limit = tune.spin_limit;
  g.wait = mode != Mode::kPreset;
  if (w_layout == DITRON_B_KN) {   // [hidden, inter] weights: the column block is 128 or 256 (a 192-column row does not split over the loading lanes)
    const bool wide = mt.block_n > 128;
    if (mt.block_m == 256) return wide ? launch_moe_gemm<GemmTile4W<256, 256, true>>(g, max_tiles, s) : launch_moe_gemm<GemmTile4W<256, 128, true>>(g, max_tiles, s);
    return wide ? launch_moe_gemm<GemmTile4W<128, 256, true>>(g, max_tiles, s) : launch_moe_gemm<GemmTile4W<128, 128, true>>(g, max_tiles, s);
  }
  if (mt.block_m == 256) {
    if (mt.block_n == 128) return launch_moe_gemm<GemmTile4W<256, 128>>(g, max_tiles, s);
    return launch_moe_gemm<TileBigDirect>(g, max_tiles, s);
  }
  // 128-row tiles: their operands are streamed (an expert's weights are read by one or two row tiles), so
  // they go through as deep a ring of LDS stages as fits
  switch (mt.block_n) {
    case 128: return launch_moe_gemm<GemmTile4W<128, 128, false, true>, 5>(g, max_tiles, s);
    case 192: return launch_moe_gemm<GemmTile4W<128, 192, false, true>, 4>(g, max_tiles, s);
    default: return launch_moe_gemm<GemmTile4W<128, 256, false, true>, 3>(g, max_tiles, s);
  }
}


// ====================================================================== MoE down-projection + ReduceScatter
// (paper: workload "MoE+ReduceScatter" of the evaluation; tensor-parallel placement.)  The activations are
// already grouped by expert (the output order of the AllGather + grouped GEMM above), so the grouped GEMM
// reads its rows in place; a top-k combine brings the rows back to token order (fp32 fma over the token's
// assignments in order, one rounding), and the reduce-scatter is the one of GEMM-ReduceScatter: the peers'
// blocks arrive in the scatter buffer, the slots are added in fp32 in slot order.
namespace ditron {

struct MoeRsPrepareParams {
  const int32_t* expert_offsets;
  int32_t* inverse_idx;    // [assignments]
  int32_t* tile_records;
  int32_t* status;
  int num_local, block_m, max_rows, max_tiles, assignments;
};

// Work-group 0: the tile list (expert after expert, no arrival stage: every row is local).  The others start
// the inverse index at "not on this rank"; the grouped GEMM that follows fills in the rows that are.
__global__ __launch_bounds__(1024) void moe_rs_prepare_kernel(const MoeRsPrepareParams p) {
  if (blockIdx.x > 0) {
    for (int f = (blockIdx.x - 1) * 1024 + threadIdx.x; f < p.assignments; f += (gridDim.x - 1) * 1024) p.inverse_idx[f] = -1;
    return;
  }
  __shared__ int s_off[kMaxLocalExperts + 1];
  __shared__ int s_first[kMaxLocalExperts + 1];
  for (int j = threadIdx.x; j <= p.num_local; j += 1024) s_off[j] = p.expert_offsets[j];
  __syncthreads();
  const int R = s_off[p.num_local];
  if (threadIdx.x == 0) {
    int tiles = 0;
    for (int j = 0; j < p.num_local; ++j) {
      s_first[j] = tiles;
      tiles += cdiv(s_off[j + 1] - s_off[j], p.block_m);
    }
    s_first[p.num_local] = tiles;
    const bool fits = R <= p.max_rows && tiles <= p.max_tiles;
    if (!fits) {
      p.status[0] = DITRON_ERR_WORKSPACE;
      p.status[2] = R;
    }
    p.tile_records[0] = fits ? tiles : 0;
  }
  __syncthreads();
  if (R > p.max_rows || s_first[p.num_local] > p.max_tiles) return;
  // one thread per tile: its expert by a walk over the (few) firsts
  for (int t = threadIdx.x; t < s_first[p.num_local]; t += 1024) {
    int j = 0;
    while (s_first[j + 1] <= t) ++j;
    int32_t* rec = p.tile_records + 1 + 4 * t;
    rec[0] = j; rec[1] = t; rec[2] = 0; rec[3] = 0;
    p.tile_records[1 + 4 * p.max_tiles + t] = s_off[j] + (t - s_first[j]) * p.block_m;
  }
}

struct MoeCombineParams {
  const __bf16* y;             // [rows, hidden] grouped by expert
  const int32_t* inverse_idx;  // [tokens * top_k]
  const float* gate;           // [tokens * top_k] or null
  __bf16* combined;            // [tokens, hidden]
  int tokens, top_k, hidden, combine_wgs;
  // own-slot flags and the emulated peers (work-groups behind the combine)
  int32_t* done;               // work-groups of the combine that have finished
  int32_t* own_flags;          // [chunks]
  const void* peer[DITRON_MAX_WORLD];
  int order[DITRON_MAX_WORLD];
  char* scatter_buf;
  int32_t* arr_flags;
  int32_t* arr_counters;
  size_t slot_bytes;
  int chunks, n_peers, num_producers, teams;
  int32_t epoch;
};

__global__ __launch_bounds__(1024) void moe_combine_kernel(const MoeCombineParams p) {
  if ((int)blockIdx.x >= p.combine_wgs) {
    const size_t chunk_bytes = p.slot_bytes / p.chunks;
    produce_chunks<1024>(
        p.n_peers * p.chunks, chunk_bytes, blockIdx.x - p.combine_wgs, p.num_producers, p.teams, p.epoch,
        [&](int i) { return (void*)(p.scatter_buf + p.order[i / p.chunks] * p.slot_bytes + (i % p.chunks) * chunk_bytes); },
        [&](int i) { return (const void*)((const char*)p.peer[p.order[i / p.chunks]] + (i % p.chunks) * chunk_bytes); },
        [&](int i) { return p.arr_flags + p.order[i / p.chunks] * p.chunks + i % p.chunks; },
        [&](int i) { return p.arr_counters + p.order[i / p.chunks] * p.chunks + i % p.chunks; });
    return;
  }
  // one lane per 8 columns of one token: top_k rows of 16 bytes in, one out
  const int vpr = p.hidden >> 3;
  const long total = (long)p.tokens * vpr;
  for (long v = (long)blockIdx.x * 1024 + threadIdx.x; v < total; v += (long)p.combine_wgs * 1024) {
    const int t = (int)(v / vpr), c = (int)(v - (long)t * vpr);
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    // the token's assignments eight at a time: positions and gates first, then every row's 16 bytes, then the
    // sum in the order j = 0, 1, ... (the loads of a batch are in flight together)
    constexpr int kBatch = 8;
    for (int j0 = 0; j0 < p.top_k; j0 += kBatch) {
      int pos[kBatch];
      float g[kBatch];
      u32x4_t x[kBatch];
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        const bool in = j0 + b < p.top_k;
        pos[b] = in ? p.inverse_idx[t * p.top_k + j0 + b] : -1;   // -1: the assignment's expert is not on this rank
        g[b] = (in && p.gate) ? p.gate[t * p.top_k + j0 + b] : 1.f;
      }
#pragma unroll
      for (int b = 0; b < kBatch; ++b)
        if (pos[b] >= 0) x[b] = __builtin_nontemporal_load((const u32x4_t*)(p.y + (size_t)pos[b] * p.hidden) + c);
#pragma unroll
      for (int b = 0; b < kBatch; ++b) {
        if (pos[b] < 0) continue;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          acc[2 * q] = __builtin_fmaf(g[b], __builtin_bit_cast(float, x[b][q] << 16), acc[2 * q]);
          acc[2 * q + 1] = __builtin_fmaf(g[b], __builtin_bit_cast(float, x[b][q] & 0xFFFF0000u), acc[2 * q + 1]);
        }
      }
    }
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    u32x4_t r;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bf16x2_t o = {(__bf16)acc[2 * q], (__bf16)acc[2 * q + 1]};
      r[q] = __builtin_bit_cast(uint32_t, o);
    }
    *((u32x4_t*)(p.combined + (size_t)t * p.hidden) + c) = r;
  }
  // the last work-group of the combine to finish raises the flags of the own slot
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(p.done, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    if (old == p.combine_wgs - 1) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(p.done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (int c = 0; c < p.chunks; ++c) flag_raise(p.own_flags + c, p.epoch);
    }
  }
}

}  // namespace ditron

extern "C" ditron_status_t ditron_moe_grouped_gemm_rs(
    const void* h, const void* w, int w_layout, const float* topk_weights, const int32_t* gather_idx,
    const int32_t* expert_offsets, void* y, int32_t* inverse_idx, int32_t* tile_records, void* combined,
    const void* const* peer_partials, void* scatter_buf, void* out, int32_t* signals, int32_t* status,
    const int* arrival_order, int tokens_per_rank, int hidden, int inter, int num_experts, int top_k,
    int num_local_experts, int max_rows, int world, int rank, int chunks_per_slot, int32_t epoch, unsigned flags,
    const ditron_tuning_t* tuning, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (tokens_per_rank <= 0 || hidden <= 0 || inter <= 0 || num_experts <= 0 || top_k <= 0 || max_rows <= 0)
    return DITRON_ERR_INVALID_ARG;
  if (num_local_experts <= 0 || num_local_experts > num_experts || chunks_per_slot < 1 ||
      tokens_per_rank % chunks_per_slot != 0)
    return DITRON_ERR_INVALID_ARG;
  if (!h || !w || !gather_idx || !expert_offsets || !y || !inverse_idx || !tile_records || !combined || !out ||
      !signals || !status)
    return DITRON_ERR_INVALID_ARG;
  if (world > 1 && !scatter_buf) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(h) || !aligned16(w) || !aligned16(y) || !aligned16(combined) || !aligned16(out) ||
      !aligned16(scatter_buf) || !aligned16(signals))
    return DITRON_ERR_INVALID_ARG;
  const Mode mode = producer_mode(flags);
  if (flags & DITRON_EPOCH_IN_MEMORY) return DITRON_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning, 1);
  if (mode == Mode::kInvalid || !tune.valid) return DITRON_ERR_INVALID_ARG;
  const bool emulate = mode == Mode::kEmulate;
  if (w_layout != DITRON_B_KN && w_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (hidden % 8 != 0 || inter % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit((size_t)max_rows, inter, 2) || !fits_32bit(hidden, inter, 2)) return DITRON_ERR_UNSUPPORTED;
  if (num_local_experts > kMaxLocalExperts) return DITRON_ERR_UNSUPPORTED;
  const long assignments = (long)world * tokens_per_rank * top_k;
  if (assignments > 0x7fffffffL) return DITRON_ERR_UNSUPPORTED;
  const int max_tiles = ditron_moe_max_tiles(max_rows, num_local_experts);
  hipStream_t s = (hipStream_t)stream;

  int order[DITRON_MAX_WORLD] = {0};
  if (emulate && world > 1) {
    if (!peer_partials) return DITRON_ERR_INVALID_ARG;
    bool seen[DITRON_MAX_WORLD] = {false};
    for (int i = 0; i < world - 1; ++i) {
      const int sr = arrival_order ? arrival_order[i] : ((rank - 1 - i) % world + world) % world;
      if (sr < 0 || sr >= world || sr == rank || seen[sr]) return DITRON_ERR_INVALID_ARG;
      seen[sr] = true;
      order[i] = sr;
      if (!peer_partials[sr] || !aligned16(peer_partials[sr])) return DITRON_ERR_INVALID_ARG;
    }
  }

  // 1. tile list; the inverse index starts at "not on this rank"
  const MoeTile mt = choose_moe_tile(moe_expected_rows((long)world * tokens_per_rank, top_k, num_experts, num_local_experts),
                                     num_local_experts, hidden);
  MoeRsPrepareParams pr{};
  pr.expert_offsets = expert_offsets;
  pr.inverse_idx = inverse_idx;
  pr.tile_records = tile_records;
  pr.status = status;
  pr.num_local = num_local_experts;
  pr.block_m = mt.block_m;
  pr.max_rows = max_rows;
  pr.max_tiles = max_tiles;
  pr.assignments = (int)assignments;
  hipLaunchKernelGGL(moe_rs_prepare_kernel, dim3(1 + (unsigned)std::min<long>(64, (assignments + 1023) / 1024)), dim3(1024), 0, s, pr);
  if (hipGetLastError() != hipSuccess) return DITRON_ERR_HIP;

  // 2. grouped GEMM y[p, :] = h[p, :] . W2_expert(p): contraction over the intermediate size, hidden columns; its
  //    work-groups of column block 0 also write the inverse index of their rows
  MoeGemmParams g{};
  g.workspace = (const char*)h;
  g.w = (const char*)w;
  g.y = (__bf16*)y;
  g.expert_offsets = expert_offsets;
  g.gather_idx = gather_idx;
  g.tile_records = tile_records;
  g.flags = signals;
  g.status = status;
  g.tokens_per_rank = tokens_per_rank;
  g.hidden = inter;
  g.inter = hidden;
  g.top_k = top_k;
  g.world = world;
  g.max_tiles = max_tiles;
  g.num_local = num_local_experts;
  g.num_xcd = 8;
  g.rows_in_place = 1;
  g.inverse_idx = inverse_idx;
  g.assignments = (int)assignments;
  g.epoch = epoch;
  g.spin_limit = tune.spin_limit;
  g.wait = 0;
  ditron_status_t st;
  if (w_layout == DITRON_B_KN) {
    const bool wide = mt.block_n > 128;
    if (mt.block_m == 256) st = wide ? launch_moe_gemm<GemmTile4W<256, 256, true>>(g, max_tiles, s) : launch_moe_gemm<GemmTile4W<256, 128, true>>(g, max_tiles, s);
    else st = wide ? launch_moe_gemm<GemmTile4W<128, 256, true>>(g, max_tiles, s) : launch_moe_gemm<GemmTile4W<128, 128, true>>(g, max_tiles, s);
  } else if (mt.block_m == 256) {
    st = mt.block_n == 128 ? launch_moe_gemm<GemmTile4W<256, 128>>(g, max_tiles, s) : launch_moe_gemm<TileBigDirect>(g, max_tiles, s);
  } else {
    // A contraction of a few K tiles: a tile is over before the ring of stages is full and costs about what a
    // work-group start costs, so 128 x 128 tiles on the two-stage loop (two work-groups fit a unit) and as many
    // work-groups as are resident at once, each walking down its share of the items (measured at the paper's
    // MoE+RS shape, whole call: 115 us with the ring tiles, 109 with these tiles, 106.5 with 512 resident
    // work-groups, 113.6 with 768; 256 x 256 tiles 108-118).
    if (inter <= 256) st = launch_moe_gemm_walk<GemmTile4W<128, 128>>(g, max_tiles, 512, s); else
    switch (mt.block_n) {
      case 128: st = launch_moe_gemm<GemmTile4W<128, 128, false, true>, 5>(g, max_tiles, s); break;
      case 192: st = launch_moe_gemm<GemmTile4W<128, 192, false, true>, 4>(g, max_tiles, s); break;
      default: st = launch_moe_gemm<GemmTile4W<128, 256, false, true>, 3>(g, max_tiles, s); break;
    }
  }
  if (st != DITRON_OK) return st;

  // 3. top-k combine into token order; the emulated peers' blocks arrive beside it
  const size_t slot_bytes = (size_t)tokens_per_rank * hidden * 2;
  MoeCombineParams c{};
  c.y = (const __bf16*)y;
  c.inverse_idx = inverse_idx;
  c.gate = topk_weights;
  c.combined = (__bf16*)combined;
  c.tokens = world * tokens_per_rank;
  c.top_k = top_k;
  c.hidden = hidden;
  // one work-group of 1024 threads per compute unit, so that the emulated peers behind them are resident from the
  // start (two such work-groups fit a unit); measured at the paper's MoE+RS shape: 256 / 384 / 512 / 2048 combine
  // work-groups -> 117 / 122 / 124 / 166 us for the whole call
  c.combine_wgs = (int)std::min<long>(256, ((long)c.tokens * (hidden / 8) + 1023) / 1024);
  c.done = signals + world;                                   // the counter word of segment 0 (unused here otherwise)
  c.own_flags = signals + 2 * world + rank * chunks_per_slot;
  for (int i = 0; i < world; ++i) {
    c.peer[i] = (emulate && i != rank && world > 1) ? peer_partials[i] : nullptr;
    c.order[i] = order[i];
  }
  c.scatter_buf = (char*)scatter_buf;
  c.arr_flags = signals + 2 * world;
  c.arr_counters = signals + 2 * world + world * chunks_per_slot;
  c.slot_bytes = slot_bytes;
  c.chunks = chunks_per_slot;
  c.n_peers = world - 1;
  const ProducerPlan pl = plan_producers((size_t)(world - 1) * slot_bytes, (world - 1) * chunks_per_slot);
  c.num_producers = (emulate && world > 1) ? std::min(pl.producers, 128) : 0;
  c.teams = std::min(pl.teams, std::max(1, c.num_producers));
  c.epoch = epoch;
  hipLaunchKernelGGL(moe_combine_kernel, dim3((unsigned)(c.combine_wgs + c.num_producers)), dim3(1024), 0, s, c);
  if (hipGetLastError() != hipSuccess) return DITRON_ERR_HIP;

  // 4. the reduction of GEMM-ReduceScatter over the `world` slots (own slot: the rank's rows of `combined`)
  const void* slots[DITRON_MAX_WORLD];
  for (int i = 0; i < world; ++i)
    slots[i] = i == rank ? (const void*)((const char*)combined + (size_t)rank * slot_bytes)
                         : (const void*)((const char*)scatter_buf + (size_t)i * slot_bytes);
  // flags preset: the peers' blocks are resident and nothing gates the sum but the stream order
  return ditron_reduce_slots(slots, out, mode == Mode::kPreset ? nullptr : signals + 2 * world, status, tokens_per_rank,
                             hidden, world, chunks_per_slot, epoch, tuning, stream);
}
