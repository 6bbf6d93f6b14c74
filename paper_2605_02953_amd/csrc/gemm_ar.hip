// GEMM + AllReduce in one-shot form, one rank's share (paper, Appendix "GEMM All-Reduce").
//
// One launch holds three kinds of work-groups.
//  * The persistent GEMM: `gemm_wgs` work-groups loop over the tiles of P = A . B (work-group g
//    takes positions g, g + G, ... of the grouped tile order), store each tile as bf16 into the
//    buffer the peers would read, and raise the tile's flag in this rank's flag array.
//  * The emulated peers (lowest indices): every other rank's partial is resident in this GPU's
//    memory, so a peer is reduced to what the consumer sees of it, its tile flags, raised in the
//    order a peer's own GEMM finishes tiles.
//  * The all-reduce consumer: work-groups draw tickets; ticket q is the tile at position q of
//    the GEMM's schedule, so tiles are reduced in the order they are finished.  The holder waits
//    for the tile's flag of every rank (one lane per rank), adds the `world` published tiles in
//    fp32 in rank order with 128-bit loads, rounds once to bf16 and writes the output tile.
//    GEMM work-groups that run out of tiles draw tickets too, so the last round of tiles is
//    reduced by the whole chip.
// The paper runs the consumer as a second kernel on compute units set aside for it and reduces
// through the switch (multimem); here there is no switch, the sum is done in software, and the
// number of compute units set aside is chosen per call from a cost model (zero when one more
// round of GEMM tiles would cost more than the overlap wins).
#include "gemm_core.h"
#include "launch.h"

namespace ditron {

struct GemmArParams {
  const void* part[DITRON_MAX_WORLD];   // every rank's published partial [M, N] bf16; part[rank] is gemm_out
  const char* a;
  const char* b;
  __bf16* gemm_out;
  __bf16* out;
  int32_t* ticket;       // next position of the reduce queue
  int32_t* done;         // work-groups that have left the queue
  int32_t* tile_flags;   // [world][ntiles]
  int32_t* status;
  int32_t* schedule;
  int m, n, k, world, rank;
  int32_t epoch;
  unsigned spin_limit;
  int num_producers, gemm_wgs, reduce_wgs;
  int group_m, num_xcd, per_xcd, npm, npn;
};

__device__ __forceinline__ void ar_tile_at(const GemmArParams& p, int position, int ntiles, int& pid_m, int& pid_n) {
  const int id = xcd_remap(position, ntiles, p.num_xcd, p.per_xcd);
  grouped_order(id, p.npm, p.npn, p.group_m, pid_m, pid_n);
}

__device__ __forceinline__ void ar_set(float (&acc)[8], const u32x4_t v) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] = __builtin_bit_cast(float, v[j] << 16);
    acc[2 * j + 1] = __builtin_bit_cast(float, v[j] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ void ar_add(float (&acc)[8], const u32x4_t v) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] += __builtin_bit_cast(float, v[j] << 16);
    acc[2 * j + 1] += __builtin_bit_cast(float, v[j] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ u32x4_t ar_pack(const float (&acc)[8]) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  u32x4_t r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    bf16x2_t v = {(__bf16)acc[2 * j], (__bf16)acc[2 * j + 1]};
    r[j] = __builtin_bit_cast(uint32_t, v);
  }
  return r;
}

// Sum of the `world` published copies of one output tile.  U vectors of 16 bytes per lane and
// rank are in flight at once (a single work-group owns its compute unit, so the loads in
// flight per lane are what fills the memory pipe).
template <class T, int WORLD, int U>
__device__ __forceinline__ void ar_reduce_tile(const GemmArParams& p, int m0, int n0) {
  const int world = WORLD > 0 ? WORLD : p.world;
  const int tile_m = min(T::BM, p.m - m0), tile_n = min(T::BN, p.n - n0);
  const int vpr = tile_n >> 3;                 // 16-byte vectors per tile row
  const int nvec = tile_m * vpr;
  const size_t ld = (size_t)p.n >> 3;          // vectors per matrix row
  const size_t base = (size_t)m0 * ld + ((size_t)n0 >> 3);
  u32x4_t* out = (u32x4_t*)p.out;
  for (int v0 = threadIdx.x; v0 < nvec; v0 += T::THREADS * U) {
    size_t off[U];
    u32x4_t x[U][WORLD > 0 ? WORLD : 1];
    float acc[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = v0 + u * T::THREADS;
      const int row = tile_n == T::BN ? v / (T::BN / 8) : v / vpr;
      const int col = v - row * vpr;
      off[u] = base + (size_t)row * ld + col;
      if (v < nvec) {
        if constexpr (WORLD > 0) {
#pragma unroll
          for (int s = 0; s < WORLD; ++s) x[u][s] = __builtin_nontemporal_load((const u32x4_t*)p.part[s] + off[u]);
        } else {
          ar_set(acc[u], __builtin_nontemporal_load((const u32x4_t*)p.part[0] + off[u]));
          for (int s = 1; s < world; ++s) ar_add(acc[u], __builtin_nontemporal_load((const u32x4_t*)p.part[s] + off[u]));
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = v0 + u * T::THREADS;
      if (v < nvec) {
        if constexpr (WORLD > 0) {
          ar_set(acc[u], x[u][0]);
#pragma unroll
          for (int s = 1; s < WORLD; ++s) ar_add(acc[u], x[u][s]);
        }
        __builtin_nontemporal_store(ar_pack(acc[u]), out + off[u]);
      }
    }
  }
}

template <class T, int WORLD>
__global__ __launch_bounds__(T::THREADS) void gemm_ar_kernel(const GemmArParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int ntiles = p.npm * p.npn;
  int wg = blockIdx.x;
  if (wg < p.num_producers) {
    // emulated peers: flag (peer, tile) for every peer, tiles in schedule order
    const int peers = p.world - 1;
    const int total = peers * ntiles;
    for (int i = wg * T::THREADS + (int)threadIdx.x; i < total; i += p.num_producers * T::THREADS) {
      int s = i % peers;
      if (s >= p.rank) ++s;
      int pid_m, pid_n;
      ar_tile_at(p, i / peers, ntiles, pid_m, pid_n);
      flag_raise(p.tile_flags + (size_t)s * ntiles + pid_m * p.npn + pid_n, p.epoch);
    }
    return;
  }
  wg -= p.num_producers;

  if (wg < p.gemm_wgs) {
    const uint32_t row_bytes = (uint32_t)p.k * 2u;
    const int M = p.m, N = p.n;
    for (int pos = wg; pos < ntiles; pos += p.gemm_wgs) {
      int pid_m, pid_n;
      ar_tile_at(p, pos, ntiles, pid_m, pid_n);
      const int m0 = pid_m * T::BM, n0 = pid_n * T::BN;
      if (p.schedule && threadIdx.x == 0) {
        int32_t* rec = p.schedule + 4 * (size_t)pos;
        rec[0] = pid_m; rec[1] = pid_n; rec[2] = wg; rec[3] = pos / p.gemm_wgs;
      }
      auto a_row = [=](int r) { return (uint32_t)min(m0 + r, M - 1) * row_bytes; };
      f32x16_t acc[T::NI][T::MI];
      if constexpr (T::B_KN) {
        gemm_mainloop<T>(acc, p.a, a_row, p.b, BColumns{(uint32_t)N * 2u, n0, N}, p.k, lds);
      } else {
        auto b_row = [=](int r) { return (uint32_t)min(n0 + r, N - 1) * row_bytes; };
        gemm_mainloop<T>(acc, p.a, a_row, p.b, b_row, p.k, lds);
      }
      store_tile_bf16<T>(acc, p.gemm_out, (size_t)p.n, m0, n0, M, N, lds);
      // every wave's stores are issued and the parked tile is no longer read: notify, and the
      // next tile may overwrite the operand stages
      __syncthreads();
      if (threadIdx.x == 0) flag_raise(p.tile_flags + (size_t)p.rank * ntiles + pid_m * p.npn + pid_n, p.epoch);
    }
  }

  // the reduce queue
  volatile int* drawn = (volatile int*)lds;
  for (;;) {
    __syncthreads();   // the previous ticket has been read by every wave
    if (threadIdx.x == 0) *drawn = __hip_atomic_fetch_add(p.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int q = *drawn;
    if (q >= ntiles) break;
    int pid_m, pid_n;
    ar_tile_at(p, q, ntiles, pid_m, pid_n);
    if ((int)threadIdx.x < p.world)
      flag_wait_lane(p.tile_flags + (size_t)threadIdx.x * ntiles, pid_m * p.npn + pid_n, 1, p.epoch, p.spin_limit, p.status);
    __syncthreads();
    ar_reduce_tile<T, WORLD, (T::BM * T::BN / 8 / T::THREADS >= 32 ? 4 : 2)>(p, pid_m * T::BM, pid_n * T::BN);
  }
  // the last work-group to leave puts the queue back to zero for the next call
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(p.done, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == p.gemm_wgs + p.reduce_wgs - 1) {
      __hip_atomic_store(p.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(p.done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <class T>
static ditron_status_t launch_ar(GemmArParams& p, hipStream_t stream) {
  const unsigned grid = (unsigned)(p.num_producers + p.gemm_wgs + p.reduce_wgs);
  auto launch = [&](auto kern) {
    if (!set_dynamic_lds((const void*)kern, T::LDS_BYTES)) return DITRON_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
    return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
  };
  if (p.world == 8) return launch(gemm_ar_kernel<T, 8>);
  return launch(gemm_ar_kernel<T, 0>);
}

int g_comm_wgs = -1;   // work-groups (= compute units) set aside for the all-reduce consumer; -1: cost model

// Compute units set aside for the consumer.  Taking X units away from the GEMM can add a round
// of tiles; leaving none means that the whole reduction runs after the GEMM.  The model takes a
// tile's MFMA time from the measured per-unit GEMM rate, lets X consumer units each stream at
// the measured single-unit rate while the GEMM runs, and reduces whatever the last round of
// tiles leaves at the chip's full streaming rate.
struct CommPlan {
  int gemm_wgs, reduce_wgs;
};
static CommPlan plan_comm(int units, int ntiles, int block_m, int block_n, int k, int world, int forced) {
  constexpr double kUnitFlops = 5.5e12;       // one compute unit inside a full-chip GEMM
  constexpr double kUnitBytes = 45e9;         // one compute unit streaming on its own work-group
  constexpr double kChipBytes = 5.0e12;       // the whole chip streaming
  const int kUnits = units / 8 * 8;
  const double t_tile = 2.0 * block_m * block_n * k / kUnitFlops;
  const double tile_bytes = (double)(world + 1) * block_m * block_n * 2;
  auto shape = [&](int x) {
    CommPlan c{};
    c.gemm_wgs = std::min(kUnits - x, ntiles);
    c.reduce_wgs = std::min(x, ntiles);
    return c;
  };
  if (forced >= 0) return shape(std::min(forced / 8 * 8, kUnits - 8));
  int best = 0;
  double best_t = 0;
  for (int x = 0; x <= kUnits / 2; x += 8) {
    const int g = std::min(kUnits - x, ntiles);
    const int rounds = cdiv(ntiles, g);
    const int last = ntiles - (rounds - 1) * g;
    const double t_gemm = rounds * t_tile;
    double t;
    if (x == 0 || rounds == 1) {
      if (x) continue;   // a single round leaves nothing to overlap
      t = t_gemm + ntiles * tile_bytes / kChipBytes;
    } else {
      const double early = (double)(ntiles - last) * tile_bytes / (x * kUnitBytes);
      t = std::max(t_gemm, t_tile + early) + last * tile_bytes / kChipBytes;
    }
    if (x == 0 || t < best_t) { best = x; best_t = t; }
  }
  return shape(best);
}

}  // namespace ditron

using namespace ditron;

extern "C" ditron_status_t ditron_set_comm_wgs(int wgs) {
  if (wgs < -1 || wgs > 192) return DITRON_ERR_INVALID_ARG;
  g_comm_wgs = wgs;
  return DITRON_OK;
}

extern "C" ditron_status_t ditron_gemm_ar(const void* a, const void* b, int b_layout, void* gemm_out,
                                          const void* const* peer_partials, void* out, int32_t* signals,
                                          int32_t* status, int32_t* schedule_out, int m, int n, int k_local,
                                          int world, int rank, int32_t epoch, unsigned flags, void* stream) {
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (m <= 0 || n <= 0 || k_local <= 0) return DITRON_ERR_INVALID_ARG;
  if (!a || !b || !gemm_out || !out || !signals || !status || out == gemm_out) return DITRON_ERR_INVALID_ARG;
  if (world > 1 && !peer_partials) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(a) || !aligned16(b) || !aligned16(gemm_out) || !aligned16(out) || !aligned16(signals))
    return DITRON_ERR_INVALID_ARG;
  const bool emulate = (flags & DITRON_EMULATE_PRODUCER) != 0;
  const bool external = (flags & DITRON_EXTERNAL_PRODUCER) != 0;
  if (emulate == external) return DITRON_ERR_INVALID_ARG;
  if ((flags & DITRON_DUMP_SCHEDULE) && !schedule_out) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (k_local % 8 != 0 || n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit(m, k_local, 2) || !fits_32bit(n, k_local, 2)) return DITRON_ERR_UNSUPPORTED;

  GemmArParams p{};
  for (int s = 0; s < world; ++s) {
    if (s == rank) {
      p.part[s] = gemm_out;
    } else {
      if (!peer_partials[s] || !aligned16(peer_partials[s]) || peer_partials[s] == out) return DITRON_ERR_INVALID_ARG;
      p.part[s] = peer_partials[s];
    }
  }
  const TileChoice tc = choose_tile(m, n, k_local);
  p.npm = cdiv(m, tc.block_m);
  p.npn = cdiv(n, tc.block_n);
  const int ntiles = p.npm * p.npn;
  // every GEMM work-group must be resident at once (the consumer waits for their tiles while it
  // holds a compute unit), so the plan is made for the compute units this device has
  int dev = 0, units = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || units < 16)
    return DITRON_ERR_HIP;
  const CommPlan cp = plan_comm(units, ntiles, tc.block_m, tc.block_n, k_local, world, g_comm_wgs);
  p.a = (const char*)a;
  p.b = (const char*)b;
  p.gemm_out = (__bf16*)gemm_out;
  p.out = (__bf16*)out;
  p.ticket = signals;
  p.done = signals + 1;
  p.tile_flags = signals + 2 * world;
  p.status = status;
  p.schedule = (flags & DITRON_DUMP_SCHEDULE) ? schedule_out : nullptr;
  p.m = m;
  p.n = n;
  p.k = k_local;
  p.world = world;
  p.rank = rank;
  p.epoch = epoch;
  p.spin_limit = g_spin_limit;
  p.num_producers = (emulate && world > 1) ? 8 : 0;
  p.gemm_wgs = cp.gemm_wgs;
  p.reduce_wgs = cp.reduce_wgs;
  p.group_m = tc.group_m;
  p.num_xcd = tc.num_xcd;
  p.per_xcd = cdiv(p.gemm_wgs, tc.num_xcd);
  const hipStream_t s = (hipStream_t)stream;
  if (b_layout == DITRON_B_KN) return tc.big ? launch_ar<TileBigKN>(p, s) : launch_ar<TileSmallKN>(p, s);
  return tc.big ? launch_ar<TileBig>(p, s) : launch_ar<TileSmall>(p, s);
}
