// GEMM + AllReduce in one-shot form, one rank's share (paper, Appendix "GEMM All-Reduce").
//
// One launch holds three kinds of work-groups.
//  * GEMM tiles: one work-group per tile of P = A . B, taken in the grouped tile order; it stores
//    the tile as bf16 into the buffer the peers would read and raises the tile's flag in this
//    rank's flag array.
//  * The emulated peers (lowest indices): every other rank's partial is resident in this GPU's
//    memory, so a peer is reduced to what the consumer sees of it, its tile flags, raised in the
//    order a peer's own GEMM finishes tiles.
//  * The all-reduce consumer: work-groups that draw tickets; ticket q is the tile at position q
//    of the tile order, so tiles are reduced in the order they are finished.  The holder waits
//    for the tile's flag of every rank (one lane per rank), adds the `world` published copies in
//    fp32 in rank order with 128-bit loads, rounds once to bf16 and writes the output tile.
// Where the consumers sit in the grid decides when they run.  When the GEMM needs more than one
// chip-wide round of tiles, X consumers follow the first round of tiles: they take X compute
// units as the first tiles retire and keep them to the end, reducing finished tiles while the
// other units compute the next ones.  Behind the last tile sit as many consumers again as the
// chip has units; they pick up compute units as the last tiles retire and the whole chip
// finishes the queue.  A tile never waits, and a consumer only waits (bounded) for tiles that
// are ahead of it in the grid, so the launch cannot deadlock.
//
// Sizing X: one work-group streams about 50 GB/s on its compute unit whatever it keeps in
// flight (measured; the whole chip reaches 5.4 TB/s only with all units streaming), so the
// reduction costs least unit-time when few units do it all along: X is the number of units
// that reduce the whole output in the time the remaining units need for the GEMM.
//
// The paper runs a persistent GEMM on a fixed set of compute units and the consumer as a second
// kernel on the rest, reducing through the switch (multimem).  Here there is no switch (the sum
// is done in software), and a persistent GEMM measured slower on this chip (its K loop ran 13 %
// slower than with one work-group per tile, which the dispatcher also load-balances).
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
  int32_t* done;         // consumers that have left the queue
  int32_t* tile_flags;   // [world][ntiles]
  // two-shot only
  __bf16* out_dst[DITRON_MAX_WORLD];      // every rank's output buffer; out_dst[rank] is `out`
  const void* reduced[DITRON_MAX_WORLD];  // emulated peers: what rank s broadcasts (only the tiles it owns are read)
  int32_t* peer_done;                     // [world]: rank s has broadcast all its tiles
  int32_t* prod_count;                    // arrival counter of the emulated peers
  int32_t* status;
  int32_t* schedule;
  int m, n, k, world, rank;
  int32_t epoch;
  unsigned spin_limit;
  int num_producers;
  int head_tiles;        // tiles ahead of the early consumers
  int early, late;       // consumers behind the first round of tiles / behind the last tile
  int peers_resident;    // flags preset: the peers' partials are complete, only the own tile flags are waited for
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
template <class T, int WORLD, int U, bool TWO>
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
        const u32x4_t r = ar_pack(acc[u]);
        if constexpr (TWO) {   // the broadcast: the reduced tile goes to every rank's output
          for (int d = 0; d < world; ++d) __builtin_nontemporal_store(r, (u32x4_t*)p.out_dst[d] + off[u]);
        } else {
          __builtin_nontemporal_store(r, out + off[u]);
        }
      }
    }
  }
}

// Two-shot, emulated peers: one tile of what a peer broadcasts lands in the local output.
template <class T>
__device__ __forceinline__ void ar_copy_tile(const GemmArParams& p, const void* src, int m0, int n0) {
  const int tile_m = min(T::BM, p.m - m0), tile_n = min(T::BN, p.n - n0);
  const int vpr = tile_n >> 3;
  const int nvec = tile_m * vpr;
  const size_t ld = (size_t)p.n >> 3;
  const size_t base = (size_t)m0 * ld + ((size_t)n0 >> 3);
  constexpr int U = 8;
  for (int v0 = threadIdx.x; v0 < nvec; v0 += T::THREADS * U) {
    size_t off[U];
    u32x4_t x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int v = v0 + u * T::THREADS;
      const int row = v / vpr;
      off[u] = base + (size_t)row * ld + (v - row * vpr);
      if (v < nvec) x[u] = __builtin_nontemporal_load((const u32x4_t*)src + off[u]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (v0 + u * T::THREADS < nvec) __builtin_nontemporal_store(x[u], (u32x4_t*)p.out + off[u]);
  }
}

// TWO: the two-shot form.  Position q of the tile order belongs to rank q % world; a rank reduces only
// its own tiles and stores each reduced tile into every rank's output; the other tiles of its output
// arrive from their owners.
template <class T, int WORLD, bool TWO>
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
    if constexpr (TWO) {
      // the peers' broadcasts: the i-th tile that is not ours is position (i / (W-1)) W + s, s the
      // (i % (W-1))-th rank other than ours
      for (int i = wg;; i += p.num_producers) {
        const int block = (i / peers) * p.world;     // first position of the block of `world` positions
        if (block >= ntiles) break;
        int s = i % peers;
        if (s >= p.rank) ++s;
        const int q = block + s;
        if (q >= ntiles) continue;
        int pid_m, pid_n;
        ar_tile_at(p, q, ntiles, pid_m, pid_n);
        ar_copy_tile<T>(p, p.reduced[s], pid_m * T::BM, pid_n * T::BN);
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(p.prod_count, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        if (old == p.num_producers - 1) {
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
          __hip_atomic_store(p.prod_count, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          for (int r = 0; r < p.world; ++r)
            if (r != p.rank) flag_raise(p.peer_done + r, p.epoch);
        }
      }
    }
    return;
  }
  wg -= p.num_producers;
  // grid: head_tiles tiles, `early` consumers, the remaining tiles, `late` consumers
  int pos = -1;
  if (wg < p.head_tiles) pos = wg;
  else if (wg >= p.head_tiles + p.early && wg < ntiles + p.early) pos = wg - p.early;

  if (pos >= 0) {
    int pid_m, pid_n;
    ar_tile_at(p, pos, ntiles, pid_m, pid_n);
    const int m0 = pid_m * T::BM, n0 = pid_n * T::BN;
    if (p.schedule && threadIdx.x == 0) {
      int32_t* rec = p.schedule + 4 * (size_t)pos;
      rec[0] = pid_m; rec[1] = pid_n; rec[2] = wg; rec[3] = 0;
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
    store_tile_bf16<T>(acc, p.gemm_out, (size_t)p.n, m0, n0, M, N, lds);
    __syncthreads();   // every wave's stores are issued: notify
    if (threadIdx.x == 0) flag_raise(p.tile_flags + (size_t)p.rank * ntiles + pid_m * p.npn + pid_n, p.epoch);
    return;
  }

  // a consumer: draw tickets until the queue is empty
  volatile int* drawn = (volatile int*)lds;
  for (;;) {
    __syncthreads();   // the previous ticket has been read by every wave
    if (threadIdx.x == 0) *drawn = __hip_atomic_fetch_add(p.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const int q = TWO ? *drawn * p.world + p.rank : *drawn;   // two-shot: only the positions this rank owns
    if (q >= ntiles) break;
    int pid_m, pid_n;
    ar_tile_at(p, q, ntiles, pid_m, pid_n);
    if ((int)threadIdx.x < p.world && (!p.peers_resident || (int)threadIdx.x == p.rank))
      flag_wait_lane(p.tile_flags + (size_t)threadIdx.x * ntiles, pid_m * p.npn + pid_n, 1, p.epoch, p.spin_limit, p.status);
    __syncthreads();
    ar_reduce_tile<T, WORLD, (T::BM * T::BN / 8 / T::THREADS >= 32 ? 4 : 2), TWO>(p, pid_m * T::BM, pid_n * T::BN);
  }
  // the last consumer to leave puts the queue back to zero for the next call
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(p.done, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (old == p.early + p.late - 1) {
      if constexpr (TWO) {
        // the output is complete when the call returns: the peers' broadcasts must have landed too
        for (int r = 0; r < p.world; ++r)
          if (r != p.rank) flag_wait_lane(p.peer_done, r, 1, p.epoch, p.spin_limit, p.status);
      }
      __hip_atomic_store(p.ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(p.done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

template <auto Kernel>
struct KernelConstant {
  static constexpr auto value = Kernel;
};

template <class T>
static ditron_status_t launch_ar(GemmArParams& p, int units, bool two_shot, hipStream_t stream) {
  const int ntiles = p.npm * p.npn;
  units = units / 8 * 8;
  p.head_tiles = std::min(ntiles, units);
  p.early = 0;
  if (ntiles > units) {
    // X units reduce while units - X compute the tiles at the per-unit MFMA rate of a full-chip GEMM:
    // balance the two.  Per GEMM tile the consumer moves (world + 1) tile-sized streams in the one-shot
    // form and 2 in the two-shot form (world reads and world writes for one tile in `world`), at ~40 GB/s
    // per unit (50 while streaming, less the waits).
    constexpr double kUnitBytes = 40e9, kUnitFlops = 5.3e12;   // (measured at table shape 3: X = 40 / 56 / 64 / 72 / 80 -> 555 / 534 / 528 / 540 / 545 us)
    const double streams = two_shot ? 2.0 : p.world + 1.0;
    const double t_reduce = streams * T::BM * T::BN * 2 / kUnitBytes;   // unit-seconds per tile
    const double t_gemm = 2.0 * T::BM * T::BN * p.k / kUnitFlops;
    const int x = (int)(units * t_reduce / (t_reduce + t_gemm) / 8 + 0.5) * 8;
    p.early = std::max(0, std::min(x, units / 2));
  }
  p.late = std::min(units, ntiles);
  const unsigned grid = (unsigned)(p.num_producers + ntiles + p.early + p.late);
  auto launch = [&](auto instance) {
    constexpr auto kern = decltype(instance)::value;
    if (!set_dynamic_lds<kern>(T::LDS_BYTES)) return DITRON_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
    return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
  };
  if (two_shot)
    return p.world == 8 ? launch(KernelConstant<gemm_ar_kernel<T, 8, true>>{}) : launch(KernelConstant<gemm_ar_kernel<T, 0, true>>{});
  return p.world == 8 ? launch(KernelConstant<gemm_ar_kernel<T, 8, false>>{}) : launch(KernelConstant<gemm_ar_kernel<T, 0, false>>{});
}

}  // namespace ditron

using namespace ditron;

static ditron_status_t gemm_ar_impl(const void* a, const void* b, int b_layout, void* gemm_out,
                                    const void* const* peer_partials, void* out, void* const* out_dsts,
                                    const void* const* peer_reduced, int32_t* signals, int32_t* status,
                                    int32_t* schedule_out, int m, int n, int k_local, int world, int rank,
                                    int32_t epoch, unsigned flags, const ditron_tuning_t* tuning, void* stream) {
  const bool two_shot = out_dsts != nullptr;

  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (m <= 0 || n <= 0 || k_local <= 0) return DITRON_ERR_INVALID_ARG;
  if (!a || !b || !gemm_out || !out || !signals || !status || out == gemm_out) return DITRON_ERR_INVALID_ARG;
  if (world > 1 && !peer_partials) return DITRON_ERR_INVALID_ARG;
  if (!aligned16(a) || !aligned16(b) || !aligned16(gemm_out) || !aligned16(out) || !aligned16(signals))
    return DITRON_ERR_INVALID_ARG;
  const Mode mode = producer_mode(flags);
  if (flags & DITRON_EPOCH_IN_MEMORY) return DITRON_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning, 1);
  if (mode == Mode::kInvalid || !tune.valid) return DITRON_ERR_INVALID_ARG;
  if (mode == Mode::kPreset && two_shot) return DITRON_ERR_UNSUPPORTED;   // the peers' broadcasts are part of the call
  const bool emulate = mode == Mode::kEmulate;
  if ((flags & DITRON_DUMP_SCHEDULE) && !schedule_out) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (k_local % 8 != 0 || n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  if (!fits_32bit(m, k_local, 2) || !fits_32bit(n, k_local, 2)) return DITRON_ERR_UNSUPPORTED;

  GemmArParams p{};
  if (two_shot) {
    for (int s = 0; s < world; ++s) {
      if (!out_dsts[s] || !aligned16(out_dsts[s]) || out_dsts[s] == gemm_out) return DITRON_ERR_INVALID_ARG;
      p.out_dst[s] = (__bf16*)out_dsts[s];
      if (s != rank && emulate) {
        if (!peer_reduced || !peer_reduced[s] || !aligned16(peer_reduced[s]) || peer_reduced[s] == out)
          return DITRON_ERR_INVALID_ARG;
        p.reduced[s] = peer_reduced[s];
      }
    }
  }
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
  int dev = 0, units = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || units < 16)
    return DITRON_ERR_HIP;
  p.a = (const char*)a;
  p.ticket = signals;
  p.done = signals + 1;
  p.b = (const char*)b;
  p.gemm_out = (__bf16*)gemm_out;
  p.out = (__bf16*)out;
  p.tile_flags = signals + 2 * world;
  p.peer_done = signals + 2 * world + (size_t)world * ntiles;
  p.prod_count = signals + 2;
  p.status = status;
  p.schedule = (flags & DITRON_DUMP_SCHEDULE) ? schedule_out : nullptr;
  p.m = m;
  p.n = n;
  p.k = k_local;
  p.world = world;
  p.rank = rank;
  p.epoch = epoch;
  p.spin_limit = tune.spin_limit;
  p.peers_resident = mode == Mode::kPreset;
  // one-shot: the emulated peers only raise flags; two-shot: they also copy the peers' broadcasts
  p.num_producers = (emulate && world > 1) ? (two_shot ? 64 : 8) : 0;
  p.group_m = tc.group_m;
  p.num_xcd = tc.num_xcd;
  p.per_xcd = tc.per_xcd;
  const hipStream_t s = (hipStream_t)stream;
  if (b_layout == DITRON_B_KN) return tc.big ? launch_ar<TileBigKN>(p, units, two_shot, s) : launch_ar<TileSmallKN>(p, units, two_shot, s);
  if (!tc.big) return launch_ar<TileSmall>(p, units, two_shot, s);
  return launch_ar<TileBigDirect>(p, units, two_shot, s);
}

extern "C" ditron_status_t ditron_gemm_ar(const void* a, const void* b, int b_layout, void* gemm_out,
                                          const void* const* peer_partials, void* out, int32_t* signals,
                                          int32_t* status, int32_t* schedule_out, int m, int n, int k_local,
                                          int world, int rank, int32_t epoch, unsigned flags,
                                          const ditron_tuning_t* tuning, void* stream) {
  return gemm_ar_impl(a, b, b_layout, gemm_out, peer_partials, out, nullptr, nullptr, signals, status, schedule_out, m, n,
                      k_local, world, rank, epoch, flags, tuning, stream);
}

extern "C" ditron_status_t ditron_gemm_ar_two_shot(const void* a, const void* b, int b_layout, void* gemm_out,
                                                   const void* const* peer_partials, void* const* out_dsts,
                                                   const void* const* peer_reduced, int32_t* signals,
                                                   int32_t* status, int32_t* schedule_out, int m, int n,
                                                   int k_local, int world, int rank, int32_t epoch, unsigned flags,
                                                   const ditron_tuning_t* tuning, void* stream) {
  if (!out_dsts || world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  return gemm_ar_impl(a, b, b_layout, gemm_out, peer_partials, out_dsts[rank], out_dsts, peer_reduced, signals, status,
                      schedule_out, m, n, k_local, world, rank, epoch, flags, tuning, stream);
}
