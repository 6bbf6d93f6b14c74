// AllGather-GEMM for decode-shaped problems (few rows, wide weight matrix), fp8 (OCP e4m3) or
// bf16 operands: C[m, n] = (gather(A) . B) * a_scale[row shard] * b_scale[col], bf16 out (no
// scales for bf16).
//
// The work is bound by streaming B once from HBM, so a work-group owns a 128-row x 32-column
// output tile and keeps many small B stages in flight: B (32 rows x 128 bytes per K tile)
// runs through a 16-deep LDS ring that is started before the shard flags are even looked at
// (B does not depend on the gather), while A (128 rows x 128 bytes per K tile, served from
// L2) uses a 5-deep ring that starts once the flags are up.  The two streams are issued by
// different waves: a wave's loads return in order, so an A load (L2 latency) queued behind a
// B load (HBM latency) would wait for it.  Waves 0-3 fetch A and compute, waves 4-7 only
// fetch B; one barrier per K tile joins them.  A K tile is 128 bytes of a row for either type:
// v_mfma_f32_16x16x128_f8f6f4 consumes 32 contiguous bytes per lane of each operand (one MFMA
// per K tile and 16 x 16 block), v_mfma_f32_16x16x32_bf16 16 bytes (two MFMAs).
#include "gemm_core.h"
#include "launch.h"

namespace ditron {

struct DecodeTile {
  static constexpr int BM = 128, BN = 32, BK = 128, NWAVES = 4, THREADS = 512;   // 4 compute waves + 4 B loaders
  static constexpr int NA = 5, NB = 16;                 // ring depths
  static constexpr int A_STAGE = BM * 128, B_STAGE = BN * 128;
  static constexpr int A_LOADS = BM / 8 / NWAVES;       // 4 wave-wide loads per wave per K tile
  static constexpr int LDS_BYTES = NA * A_STAGE + NB * B_STAGE;
  // loads of a wave that may still be in flight when tile kt is needed: the younger tiles of its ring
  static constexpr int PENDING_A = (NA - 2) * A_LOADS, PENDING_B = NB - 2;
};

typedef int i32x8_t __attribute__((ext_vector_type(8)));

struct AgGemmDecodeParams {
  const void* shard[DITRON_MAX_WORLD];
  int order[DITRON_MAX_WORLD];
  char* workspace;
  const char* b;
  __bf16* c;
  const float* a_scales;
  const float* b_scales;
  int32_t* flags;
  int32_t* arrivals;
  int32_t* status;
  int32_t* schedule;
  int m_per_rank, m, n, k, world, rank, nnodes;   // k in elements
  int32_t epoch;
  int32_t* epoch_word;   // if set: the call's epoch is 1 + this word, which the last work-group to finish advances
  int32_t* finished;     // ... counting the work-groups that are done
  int num_producers, teams;
  unsigned spin_limit;
  int wait;   // 0: every shard is resident, the flags are not looked at
  int timing; // schedule records hold time stamps instead
  int group_m, num_xcd, per_xcd, npm, npn;
  // split-K kernel
  int splits, kt_per_split;   // K splits per output tile; 128-byte K tiles per split
  char* partials;             // [tile][split][BM x BN] words of 8 bytes (fp32 value, epoch), in the lanes' own order
};

template <bool BF16>
__global__ __launch_bounds__(DecodeTile::THREADS) void ag_gemm_decode_kernel(const AgGemmDecodeParams p) {
  typedef DecodeTile T;
  const int K = p.k * (BF16 ? 2 : 1);   // bytes per row of A and of B
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  if ((int)blockIdx.x < p.num_producers) {
    const size_t shard_bytes = (size_t)p.m_per_rank * K;
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
  pid_m = p.nnodes > 1 ? tile_row_across_nodes(pid_m, p.m, p.rank, p.world, p.nnodes, T::BM, kOrderGather)
                       : (pid_m + cdiv(p.m_per_rank * p.rank, T::BM)) % p.npm;
  const int m0 = pid_m * T::BM, n0 = pid_n * T::BN;
  const int rank_beg = m0 / p.m_per_rank;
  const int rank_end = (min(m0 + T::BM, p.m) - 1) / p.m_per_rank;
  if (p.schedule && !p.timing && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * (size_t)wg;
    rec[0] = pid_m; rec[1] = pid_n; rec[2] = rank_beg; rec[3] = rank_end;
  }

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int kt_all = (K + T::BK - 1) / T::BK;
  char* lds_a = lds;
  char* lds_b = lds + T::NA * T::A_STAGE;

  // per-lane source addresses (K tile 0) and the byte offset of the lane's chunk in a K tile
  const char* a_ptr[T::A_LOADS];
  int a_kc[T::A_LOADS];
#pragma unroll
  for (int i = 0; i < T::A_LOADS; ++i) {
    const int r = (wave * T::A_LOADS + i) * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz128(r);
    a_kc[i] = c * 16;
    a_ptr[i] = p.workspace + (size_t)min(m0 + r, p.m - 1) * K + c * 16;
  }
  const bool loader = wave >= T::NWAVES;        // waves 4-7 stream B, waves 0-3 stream A and compute
  const int lw = wave - T::NWAVES;
  const int rb = (loader ? lw : 0) * 8 + (lane >> 3);
  const int cb = (lane & 7) ^ swz128(rb);
  const int b_kc = cb * 16;
  const char* b_ptr = p.b + (size_t)min(n0 + rb, p.n - 1) * K + cb * 16;

  // tile indices past the end fetch 16 constant bytes into a free stage: the number of loads per
  // iteration stays fixed, which is what the in-order wait counts below rely on
  auto issue_a = [&](int kt) {
    const int kte = min(kt, kt_all - 1);
    char* stage = lds_a + (kt % T::NA) * T::A_STAGE;
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
      const char* src = a_ptr[i] + (size_t)kte * T::BK;
      if (kt >= kt_all || kte * T::BK + a_kc[i] >= K) src = (const char*)&kZeroChunk;
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(stage + (wave * T::A_LOADS + i) * 1024), 16, 0, 0);
    }
  };
  auto issue_b = [&](int kt) {
    const int kte = min(kt, kt_all - 1);
    char* stage = lds_b + (kt % T::NB) * T::B_STAGE;
    const char* src = b_ptr + (size_t)kte * T::BK;
    if (kt >= kt_all || kte * T::BK + b_kc >= K) src = (const char*)&kZeroChunk;
    __builtin_amdgcn_global_load_lds(src, DITRON_LDS(stage + lw * 1024), 16, 0, 0);
  };

  // wave 0 looks at the flags; the loaders start B at once (it does not depend on the gather)
  if (wave == 0 && p.wait) flag_wait_wave(p.flags, rank_beg, rank_end - rank_beg + 1, p.epoch, p.spin_limit, p.status);
  if (loader) {
#pragma unroll 1
    for (int kt = 0; kt < T::NB - 1; ++kt) issue_b(kt);
  }
  barrier_no_drain();                           // flags seen by wave 0 -> A may be read by everyone
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  if (loader) {
#pragma unroll 1
    for (int kt = 0; kt < kt_all; ++kt) {
      // B(kt) has landed once at most PENDING_B younger loads of this wave are outstanding
      __builtin_amdgcn_s_waitcnt(0x0F70 | (T::PENDING_B & 0xF) | ((T::PENDING_B >> 4) << 14));
      barrier_no_drain();
      issue_b(kt + T::NB - 1);                  // into the stage every wave finished reading before this barrier
    }
    wait_vmcnt0();                              // the redundant tail loads land before the LDS is handed back
    return;
  }
#pragma unroll
  for (int j = 0; j < T::NA - 1; ++j) issue_a(j);

  f32x4_t acc[2][2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) acc[nb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int l16 = lane & 15, g = lane >> 4;
  const int sw = swz128(l16);
  const int off0 = ((2 * g) ^ sw) * 16, off1 = ((2 * g + 1) ^ sw) * 16;

#pragma unroll 1
  for (int kt = 0; kt < kt_all; ++kt) {
    // A(kt) has landed once at most PENDING_A younger loads of this wave are outstanding
    __builtin_amdgcn_s_waitcnt(0x0F70 | (T::PENDING_A & 0xF) | ((T::PENDING_A >> 4) << 14));
    barrier_no_drain();
    issue_a(kt + T::NA - 1);
    const char* sa = lds_a + (kt % T::NA) * T::A_STAGE + (wave * 32 + l16) * 128;
    const char* sb = lds_b + (kt % T::NB) * T::B_STAGE + l16 * 128;
    if constexpr (BF16) {
      // MFMA j of the K tile takes k = 32 j + 8 g .. + 7 of the lane's row: 16-byte chunk 4 j + g
      bf16x8_t af[2][2], bf[2][2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 2; ++j) af[mb][j] = *(const bf16x8_t*)(sa + mb * 16 * 128 + (((4 * j + g) ^ sw) * 16));
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int j = 0; j < 2; ++j) bf[nb][j] = *(const bf16x8_t*)(sb + nb * 16 * 128 + (((4 * j + g) ^ sw) * 16));
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
            acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[nb][j], af[mb][j], acc[nb][mb], 0, 0, 0);
    } else {
      i32x8_t af[2], bf[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const u32x4_t lo = *(const u32x4_t*)(sa + mb * 16 * 128 + off0);
        const u32x4_t hi = *(const u32x4_t*)(sa + mb * 16 * 128 + off1);
        af[mb] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const u32x4_t lo = *(const u32x4_t*)(sb + nb * 16 * 128 + off0);
        const u32x4_t hi = *(const u32x4_t*)(sb + nb * 16 * 128 + off1);
        bf[nb] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          acc[nb][mb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[nb], af[mb], acc[nb][mb], 0, 0, 0, 0, 0, 0);
    }
  }
  // drain the redundant tail loads before the LDS is handed back
  wait_vmcnt0();

#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int m = m0 + wave * 32 + mb * 16 + l16;
    if (m >= p.m) continue;
    const float rs = p.a_scales ? p.a_scales[m / p.m_per_rank] : 1.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int n = n0 + nb * 16 + g * 4;
      if (n >= p.n) continue;   // n is a multiple of 4 and p.n of 8: all four columns are inside
      float x[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) x[v] = acc[nb][mb][v] * rs * (p.b_scales ? p.b_scales[n + v] : 1.f);
      bf16x4_t o = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
      *(bf16x4_t*)(p.c + (size_t)m * p.n + n) = o;
    }
  }
}


// ------------------------------------------------------------------ split-K form
// The 128 x 32 tile above makes every work-group stream all of A through its compute unit (1 MiB
// for 256 KiB of B at the decode shape), and the path from the L2 into a compute unit is what bounds
// it.  Here a work-group owns a BM x BN tile over 1/S of the contraction: per 128-byte K tile it
// loads BM + BN rows instead of 128 + 32, so with 128 x 128 tiles and S = 4 a unit moves 512 KiB
// where the form above moves 1.25 MiB.  The S partial tiles (fp32, written in the lanes' own order so
// that every store and load is a contiguous KiB per wave) meet in memory: each work-group stores its
// partial, then draws a ticket from the tile's counter; the one that draws the last ticket adds the S
// partials in split order 0..S-1 (its own from registers, so the order and hence the bits do not depend
// on who came last), applies the scales and writes C.  No work-group waits for another, so the grid may
// be of any size.  Waves 0-3 fetch A and compute, waves 4-7 fetch B, one barrier per K tile, as above.
// BM = 16 is the per-shard form: a tile is one shard's rows and waits for that shard's flag only.
template <int BM_, int BN_>
struct SplitKTile {
  static constexpr int BM = BM_, BN = BN_, BK = 128, THREADS = 512;
  static constexpr int WM = BM >= 128 ? 2 : 1, WN = 4 / WM;          // the four computing waves as WM x WN
  static constexpr int WTM = BM / WM, WTN = BN / WN;
  static constexpr int MB = WTM / 16, NB = WTN / 16;                  // 16 x 16 blocks per wave
  static constexpr int A_STAGE = BM * 128, B_STAGE = BN * 128;
  static constexpr int A_GROUPS = BM / 8;                             // wave-wide loads (8 rows each) per K tile of A
  static constexpr int A_LOADS = (A_GROUPS + 3) / 4;                  // per computing wave
  static constexpr int B_LOADS = BN / 32;                             // per loading wave
  static constexpr int NA = BM >= 128 ? 4 : 6;                        // ring depths: A comes from the L2, B from HBM
  static constexpr int NBR_FIT = (160 * 1024 - NA * A_STAGE) / B_STAGE;
  static constexpr int NBR = NBR_FIT > 10 ? 10 : NBR_FIT;
  static constexpr int LDS_BYTES = NA * A_STAGE + NBR * B_STAGE;
  static constexpr int PENDING_A = (NA - 2) * A_LOADS, PENDING_B = (NBR - 2) * B_LOADS;
  static constexpr int TILE_WORDS = BM * BN;                          // fp32 words of one partial tile
  static_assert(MB >= 1 && NB >= 1 && PENDING_B <= 63 && PENDING_A <= 63, "tile shape");
};

template <bool BF16, class T>
__device__ __forceinline__ void splitk_work_group(const AgGemmDecodeParams& p, const int32_t epoch, char* lds) {
  const int K = p.k * (BF16 ? 2 : 1);   // bytes per row of A and of B
  if ((int)blockIdx.x < p.num_producers) {
    const size_t shard_bytes = (size_t)p.m_per_rank * K;
    produce_chunks<T::THREADS>(
        p.world, shard_bytes, blockIdx.x, p.num_producers, p.teams, epoch,
        [&](int i) { return (void*)(p.workspace + (size_t)p.order[i] * shard_bytes); },
        [&](int i) { return p.shard[p.order[i]]; }, [&](int i) { return p.flags + p.order[i]; },
        [&](int i) { return p.arrivals + p.order[i]; });
    return;
  }
  // work-group -> (tile, split): tiles are dealt to the chiplets in turn and the S splits of a tile are S
  // consecutive work-groups of one chiplet, so the partials of a tile meet in one L2
  const int wg = blockIdx.x - p.num_producers;
  const int slot = wg / p.num_xcd;
  const int tile = (slot / p.splits) * p.num_xcd + wg % p.num_xcd, ks = slot % p.splits;
  const int ntiles = p.npm * p.npn;
  if (tile >= ntiles) return;
  const TileOrder order{p.npm, p.npn, p.group_m, 0, 0};
  const TileSpan t = tile_of_workgroup(tile, order, kOrderGather, p.m, p.m_per_rank, p.rank, p.world, p.nnodes, T::BM);
  const int m0 = t.pid_m * T::BM, n0 = t.pid_n * T::BN;
  const unsigned long long ts_start = p.timing ? wall_clock64() : 0;
  unsigned long long ts_wait = 0, ts_ready = 0;
  if (p.schedule && !p.timing && threadIdx.x == 0) {
    int32_t* rec = p.schedule + 4 * ((size_t)tile * p.splits + ks);
    rec[0] = t.pid_m; rec[1] = t.pid_n; rec[2] = t.first; rec[3] = t.last;
  }

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int kt_begin = ks * p.kt_per_split;
  const int kt_n = min((K + T::BK - 1) / T::BK, kt_begin + p.kt_per_split) - kt_begin;   // >= 1 by the host's choice of S
  char* lds_a = lds;
  char* lds_b = lds + T::NA * T::A_STAGE;
  const bool loader = wave >= 4;
  const int lw = wave - 4;

  // per-lane source addresses at this split's first K tile, and the byte offset of the lane's chunk in a K tile
  const char* src_ptr[T::A_LOADS > T::B_LOADS ? T::A_LOADS : T::B_LOADS];
  int src_kc[T::A_LOADS > T::B_LOADS ? T::A_LOADS : T::B_LOADS];
  if (loader) {
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
      const int r = (lw * T::B_LOADS + i) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz128(r);
      src_kc[i] = c * 16;
      src_ptr[i] = p.b + (size_t)min(n0 + r, p.n - 1) * K + (size_t)kt_begin * T::BK + c * 16;
    }
  } else {
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
      const int r = (wave * T::A_LOADS + i) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz128(r);
      src_kc[i] = c * 16;
      src_ptr[i] = p.workspace + (size_t)min(m0 + r, p.m - 1) * K + (size_t)kt_begin * T::BK + c * 16;
    }
  }
  // K tile i of this split (requests past its end fetch 16 constant bytes into a free stage: the number of
  // loads per iteration stays fixed, which the in-order wait counts rely on, and nothing more is asked of
  // memory: re-reading real tiles there kept 5 stale tiles per unit in the queues the partial exchange needs)
  auto issue_a = [&](int i) {
    const int kt = min(i, kt_n - 1);
    char* stage = lds_a + (i % T::NA) * T::A_STAGE;
#pragma unroll
    for (int j = 0; j < T::A_LOADS; ++j) {
      const int group = wave * T::A_LOADS + j;
      if (group >= T::A_GROUPS) break;   // fewer row groups than waves (16-row tiles)
      const char* src = src_ptr[j] + (size_t)kt * T::BK;
      if (i >= kt_n || (kt_begin + kt) * T::BK + src_kc[j] >= K) src = (const char*)&kZeroChunk;
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(stage + group * 1024), 16, 0, 0);
    }
  };
  auto issue_b = [&](int i) {
    const int kt = min(i, kt_n - 1);
    char* stage = lds_b + (i % T::NBR) * T::B_STAGE;
#pragma unroll
    for (int j = 0; j < T::B_LOADS; ++j) {
      const char* src = src_ptr[j] + (size_t)kt * T::BK;
      if (i >= kt_n || (kt_begin + kt) * T::BK + src_kc[j] >= K) src = (const char*)&kZeroChunk;
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(stage + (lw * T::B_LOADS + j) * 1024), 16, 0, 0);
    }
  };

  // wave 0 looks at the flags; the loaders start B at once (it does not depend on the gather)
  // (two tiles only before the barrier: a deeper burst fills the unit's miss queue and the first loads
  // of A, issued after the barrier, would wait behind it)
  if (p.timing) ts_wait = wall_clock64();
  if (wave == 0 && p.wait) flag_wait_wave(p.flags, t.first, t.last - t.first + 1, epoch, p.spin_limit, p.status);
  if (p.timing) ts_ready = wall_clock64();
  if (loader) {
    issue_b(0);
    issue_b(1);
  }
  barrier_no_drain();                           // flags seen by wave 0 -> A may be read by everyone
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  f32x4_t acc[T::NB][T::MB];
#pragma unroll
  for (int nb = 0; nb < T::NB; ++nb)
#pragma unroll
    for (int mb = 0; mb < T::MB; ++mb) acc[nb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const int wm = loader ? 0 : wave / T::WN, wn = loader ? 0 : wave % T::WN;
  const int l16 = lane & 15, g = lane >> 4;

  if (loader) {
#pragma unroll 1
    for (int i = 2; i < T::NBR - 1; ++i) issue_b(i);
#pragma unroll 1
    for (int i = 0; i < kt_n; ++i) {
      // B(i) has landed once at most PENDING_B younger loads of this wave are outstanding
      __builtin_amdgcn_s_waitcnt(0x0F70 | (T::PENDING_B & 0xF) | ((T::PENDING_B >> 4) << 14));
      barrier_no_drain();
      issue_b(i + T::NBR - 1);                  // into the stage every wave finished reading before this barrier
    }
  } else {
#pragma unroll
    for (int j = 0; j < T::NA - 1; ++j) issue_a(j);
    const int sw = swz128(l16);
    const int off0 = ((2 * g) ^ sw) * 16, off1 = ((2 * g + 1) ^ sw) * 16;
#pragma unroll 1
    for (int i = 0; i < kt_n; ++i) {
      __builtin_amdgcn_s_waitcnt(0x0F70 | (T::PENDING_A & 0xF) | ((T::PENDING_A >> 4) << 14));
      barrier_no_drain();
      issue_a(i + T::NA - 1);
      const char* sa = lds_a + (i % T::NA) * T::A_STAGE + (wm * T::WTM + l16) * 128;
      const char* sb = lds_b + (i % T::NBR) * T::B_STAGE + (wn * T::WTN + l16) * 128;
      if constexpr (BF16) {
        // MFMA j of the K tile takes k = 32 j + 8 g .. + 7 of the lane's row: 16-byte chunk 4 j + g
        bf16x8_t af[T::MB][2], bf[T::NB][2];
#pragma unroll
        for (int mb = 0; mb < T::MB; ++mb)
#pragma unroll
          for (int j = 0; j < 2; ++j) af[mb][j] = *(const bf16x8_t*)(sa + mb * 16 * 128 + (((4 * j + g) ^ sw) * 16));
#pragma unroll
        for (int nb = 0; nb < T::NB; ++nb)
#pragma unroll
          for (int j = 0; j < 2; ++j) bf[nb][j] = *(const bf16x8_t*)(sb + nb * 16 * 128 + (((4 * j + g) ^ sw) * 16));
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int nb = 0; nb < T::NB; ++nb)
#pragma unroll
            for (int mb = 0; mb < T::MB; ++mb)
              acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf[nb][j], af[mb][j], acc[nb][mb], 0, 0, 0);
      } else {
        i32x8_t af[T::MB], bf[T::NB];
#pragma unroll
        for (int mb = 0; mb < T::MB; ++mb) {
          const u32x4_t lo = *(const u32x4_t*)(sa + mb * 16 * 128 + off0);
          const u32x4_t hi = *(const u32x4_t*)(sa + mb * 16 * 128 + off1);
          af[mb] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        }
#pragma unroll
        for (int nb = 0; nb < T::NB; ++nb) {
          const u32x4_t lo = *(const u32x4_t*)(sb + nb * 16 * 128 + off0);
          const u32x4_t hi = *(const u32x4_t*)(sb + nb * 16 * 128 + off1);
          bf[nb] = i32x8_t{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
        }
#pragma unroll
        for (int nb = 0; nb < T::NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < T::MB; ++mb)
            acc[nb][mb] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bf[nb], af[mb], acc[nb][mb], 0, 0, 0, 0, 0, 0);
      }
    }
  }
  // the redundant tail loads land before the LDS is used for anything else
  wait_vmcnt0();

  constexpr int BLOCKS = T::MB * T::NB;
  if (p.splits > 1) {
    // The S partial tiles meet in memory, flag-in-data (the low-latency protocol of the paper's kernel
    // library, applied where this kernel's latency is): every 8-byte word carries one fp32 value and the
    // call's epoch, so a reader needs no counter and no fence; it reads the words it needs and reads them
    // again until they all carry this call's epoch.  Stores are written through and loads go past the
    // caches (sc0 sc1 on both), so this holds wherever the dispatcher put the work-groups.
    constexpr int kCoherent = 17;                                  // sc0 | sc1 on the load / store
    constexpr int UNITS = 4 * BLOCKS;                              // (wave, block) pieces per partial tile, 2 KiB each
    const size_t tile_bytes = (size_t)T::TILE_WORDS * 2 * sizeof(float);
    const __amdgpu_buffer_rsrc_t part = __builtin_amdgcn_make_buffer_rsrc(
        (char*)p.partials + (size_t)tile * p.splits * tile_bytes, 0, (int)(p.splits * tile_bytes), 0x00020000);
    const uint32_t tag = (uint32_t)epoch;
    // This work-group finishes 1/S of the tile: pieces [u_lo, u_hi).  Its own partial of those pieces never
    // leaves the compute unit: the wave that holds it parks it in the (now idle) operand rings.
    const int u_lo = ks * UNITS / p.splits, u_hi = (ks + 1) * UNITS / p.splits;
    __syncthreads();   // every wave is past its last fragment read
    if (!loader) {
      // in the lanes' own order: half h of block (nb, mb) of wave w is 64 lanes x 16 contiguous bytes
#pragma unroll
      for (int nb = 0; nb < T::NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < T::MB; ++mb) {
          const int blk = nb * T::MB + mb, u = wave * BLOCKS + blk;
          if (u >= u_lo && u < u_hi) {
            *(f32x4_t*)(lds + (u - u_lo) * 1024 + lane * 16) = acc[nb][mb];
          } else {
            const u32x4_t v = __builtin_bit_cast(u32x4_t, acc[nb][mb]);
            const int off = ((ks * 4 + wave) * BLOCKS + blk) * 2048 + lane * 16;
            __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{v[0], tag, v[1], tag}, part, off, 0, kCoherent);
            __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{v[2], tag, v[3], tag}, part, off + 1024, 0, kCoherent);
          }
        }
    }
    __syncthreads();   // the parked partial is there
    // The pieces are dealt to the eight waves; the S partials of a piece are added in split order, whoever
    // wrote them last.  The other splits of the tile are neighbours in the grid: work-groups are dispatched in
    // index order, so whenever some of them are polling here the rest is running or next in line.
    for (int u = u_lo + wave; u < u_hi; u += 8) {
      const f32x4_t own = *(const f32x4_t*)(lds + (u - u_lo) * 1024 + lane * 16);
      u32x4_t v[8][2];
      unsigned polls = 0;
      for (;;) {
        bool ok = true;
#pragma unroll
        for (int sp = 0; sp < 8; ++sp)
          if (sp < p.splits && sp != ks) {
            v[sp][0] = __builtin_amdgcn_raw_buffer_load_b128(part, (sp * UNITS + u) * 2048 + lane * 16, 0, kCoherent);
            v[sp][1] = __builtin_amdgcn_raw_buffer_load_b128(part, (sp * UNITS + u) * 2048 + 1024 + lane * 16, 0, kCoherent);
          }
#pragma unroll
        for (int sp = 0; sp < 8; ++sp)
          if (sp < p.splits && sp != ks) ok = ok && v[sp][0][1] == tag && v[sp][0][3] == tag && v[sp][1][1] == tag && v[sp][1][3] == tag;
        if (__all(ok)) break;
        if (++polls >= p.spin_limit) {
          if (lane == 0) {
            p.status[1] = 4 * p.world + tile;
            p.status[0] = DITRON_ERR_TIMEOUT;
          }
          break;
        }
      }
      f32x4_t tot;
#pragma unroll
      for (int sp = 0; sp < 8; ++sp)
        if (sp < p.splits) {
          const f32x4_t lo = __builtin_bit_cast(f32x4_t, v[sp][0]), hi = __builtin_bit_cast(f32x4_t, v[sp][1]);
          const f32x4_t x = sp == ks ? own : __builtin_shufflevector(lo, hi, 0, 2, 4, 6);
          tot = sp == 0 ? x : tot + x;
        }
      const int w = u / BLOCKS, blk = u % BLOCKS, nb = blk / T::MB, mb = blk % T::MB;
      const int m = m0 + (w / T::WN) * T::WTM + mb * 16 + l16;
      const int n = n0 + (w % T::WN) * T::WTN + nb * 16 + g * 4;
      if (m >= p.m || n >= p.n) continue;   // n is a multiple of 4 and p.n of 8: all four columns are inside
      const float rs = p.a_scales ? p.a_scales[m / p.m_per_rank] : 1.f;
      float x[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) x[q] = tot[q] * rs * (p.b_scales ? p.b_scales[n + q] : 1.f);
      bf16x4_t o = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
      *(bf16x4_t*)(p.c + (size_t)m * p.n + n) = o;
    }
    if (p.timing && threadIdx.x == 0) {
      int32_t* rec = p.schedule + 4 * ((size_t)tile * p.splits + ks);
      rec[0] = (int32_t)(ts_start & 0x7fffffff); rec[1] = (int32_t)(ts_wait & 0x7fffffff);
      rec[2] = (int32_t)(ts_ready & 0x7fffffff); rec[3] = (int32_t)(wall_clock64() & 0x7fffffff);
    }
    return;
  }
  if (p.timing && threadIdx.x == 0) {   // the contraction was not split: stamped before the stores below are issued
    int32_t* rec = p.schedule + 4 * ((size_t)tile * p.splits + ks);
    rec[0] = (int32_t)(ts_start & 0x7fffffff); rec[1] = (int32_t)(ts_wait & 0x7fffffff);
    rec[2] = (int32_t)(ts_ready & 0x7fffffff); rec[3] = (int32_t)(wall_clock64() & 0x7fffffff);
  }
  if (loader) return;

#pragma unroll
  for (int mb = 0; mb < T::MB; ++mb) {
    const int m = m0 + wm * T::WTM + mb * 16 + l16;
    if (m >= p.m) continue;
    const float rs = p.a_scales ? p.a_scales[m / p.m_per_rank] : 1.f;
#pragma unroll
    for (int nb = 0; nb < T::NB; ++nb) {
      const int n = n0 + wn * T::WTN + nb * 16 + g * 4;
      if (n >= p.n) continue;   // n is a multiple of 4 and p.n of 8: all four columns are inside
      float x[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) x[v] = acc[nb][mb][v] * rs * (p.b_scales ? p.b_scales[n + v] : 1.f);
      bf16x4_t o = {(__bf16)x[0], (__bf16)x[1], (__bf16)x[2], (__bf16)x[3]};
      *(bf16x4_t*)(p.c + (size_t)m * p.n + n) = o;
    }
  }
}

// The epoch of a call is a launch argument, or, for callers that record the launch once and replay it (a HIP
// graph), one more than a word in memory: every work-group reads the word when it starts, and the last one to
// finish (they count themselves) writes the new epoch there, after every other work-group has read the old one.
template <bool BF16, class T>
__global__ __launch_bounds__(T::THREADS) void ag_gemm_splitk_kernel(const AgGemmDecodeParams p) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  int32_t epoch = p.epoch;
  if (p.epoch_word)
    epoch = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.epoch_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) + 1;
  splitk_work_group<BF16, T>(p, epoch, lds);
  if (p.epoch_word) {
    __syncthreads();
    if (threadIdx.x == 0) {
      const int old = __hip_atomic_fetch_add(p.finished, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (int)gridDim.x - 1) {
        __hip_atomic_store(p.finished, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(p.epoch_word, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

}  // namespace ditron

using namespace ditron;

template <bool BF16, class T>
static ditron_status_t launch_splitk(AgGemmDecodeParams& p, hipStream_t stream) {
  if (!set_dynamic_lds<ag_gemm_splitk_kernel<BF16, T>>(T::LDS_BYTES)) return DITRON_ERR_HIP;
  const int per_xcd = cdiv(p.npm * p.npn, p.num_xcd) * p.splits;   // work-groups of one chiplet
  const unsigned grid = (unsigned)(p.num_producers + per_xcd * p.num_xcd);
  hipLaunchKernelGGL((ag_gemm_splitk_kernel<BF16, T>), dim3(grid), dim3(T::THREADS), T::LDS_BYTES, stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}

extern "C" ditron_status_t ditron_ag_gemm_decode(const void* const* a_shards, const void* b, int b_layout, void* c,
                                                 const float* a_scales, const float* b_scales, void* workspace,
                                                 int32_t* signals, int32_t* status, int32_t* schedule_out,
                                                 const int* arrival_order, int m_per_rank, int n, int k, int world,
                                                 int rank, int dtype, int32_t epoch, unsigned flags,
                                                 const ditron_tuning_t* tuning, void* stream) {
  // pointer / enum / mode checks were done by ditron_ag_gemm
  const Tuning tune = resolve_tuning(tuning, world);
  const bool bf16 = dtype == DITRON_BF16;
  if (b_layout != DITRON_B_NK) return DITRON_ERR_UNSUPPORTED;
  if (k % (bf16 ? 8 : 16) != 0 || n % 8 != 0) return DITRON_ERR_UNSUPPORTED;
  const bool emulate = (flags & DITRON_EMULATE_PRODUCER) != 0;
  AgGemmDecodeParams p{};
  for (int i = 0; i < world; ++i) {
    p.shard[i] = emulate ? a_shards[i] : nullptr;
    p.order[i] = arrival_order ? arrival_order[i] : (rank + i) % world;
  }
  p.workspace = (char*)workspace;
  p.b = (const char*)b;
  p.c = (__bf16*)c;
  p.a_scales = bf16 ? nullptr : a_scales;
  p.b_scales = bf16 ? nullptr : b_scales;
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
  if (flags & DITRON_EPOCH_IN_MEMORY) {
    const size_t words = ditron_signal_words(world, 1);
    p.epoch_word = signals + words - 1;
    p.finished = signals + words - 2;
  }
  p.spin_limit = tune.spin_limit;
  p.wait = producer_mode(flags) != Mode::kPreset;
  const size_t a_bytes = (size_t)p.m * k * (bf16 ? 2 : 1);
  const DecodePlan plan = plan_decode(p.m, n, k * (bf16 ? 2 : 1), tune.decode_variant);
  if (p.nnodes > 1 && !node_order_is_bijection(p.m, plan.block_m, world, p.nnodes, rank, kOrderGather))
    return DITRON_ERR_UNSUPPORTED;
  const TileChoice tc = choose_tile_decode(p.m, n, k);
  p.group_m = tc.group_m;
  p.num_xcd = tc.num_xcd;
  p.per_xcd = tc.per_xcd;
  const ProducerPlan pl = plan_producers(a_bytes, world);
  p.num_producers = emulate ? pl.producers : 0;
  p.teams = pl.teams;
  p.npm = cdiv(p.m, plan.block_m);
  p.npn = cdiv(p.n, plan.block_n);
  p.splits = plan.splits;
  p.kt_per_split = plan.kt_per_split;
  p.partials = (char*)workspace + align256(a_bytes);
  const hipStream_t s = (hipStream_t)stream;
  switch (plan.variant) {
    case 2: return bf16 ? launch_splitk<true, SplitKTile<128, 128>>(p, s) : launch_splitk<false, SplitKTile<128, 128>>(p, s);
    case 3: return bf16 ? launch_splitk<true, SplitKTile<128, 64>>(p, s) : launch_splitk<false, SplitKTile<128, 64>>(p, s);
    case 4: return bf16 ? launch_splitk<true, SplitKTile<16, 128>>(p, s) : launch_splitk<false, SplitKTile<16, 128>>(p, s);
    default: break;
  }
  if (p.epoch_word) return DITRON_ERR_UNSUPPORTED;   // the 128 x 32 kernel takes its epoch as an argument only
  if (!(bf16 ? set_dynamic_lds<ag_gemm_decode_kernel<true>>(DecodeTile::LDS_BYTES)
             : set_dynamic_lds<ag_gemm_decode_kernel<false>>(DecodeTile::LDS_BYTES)))
    return DITRON_ERR_HIP;
  auto kern = bf16 ? ag_gemm_decode_kernel<true> : ag_gemm_decode_kernel<false>;
  const unsigned grid = (unsigned)(p.num_producers + p.npm * p.npn);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(DecodeTile::THREADS), DecodeTile::LDS_BYTES, s, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}
