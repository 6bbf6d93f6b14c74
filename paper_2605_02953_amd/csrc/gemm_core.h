// bf16 MFMA tile engine for gfx950: C_tile[BM,BN] (fp32) += A_tile[BM,K] . B_tile[BN,K]^T.
//
// Both operands are read as rows that are contiguous along the contraction dimension.
// A K-slice of BK=64 elements of BM + BN rows is staged in LDS as 128-byte rows (one cache
// line per row) whose eight 16-byte chunks are XOR-swizzled by the row index; the staging
// uses the direct global->LDS load, which needs no registers.  Each wave owns a WTM x WTN sub-tile and
// feeds v_mfma_f32_32x32x16_bf16 from 128-bit LDS reads.  The instruction's row operand is
// taken from the B rows and its column operand from the A rows, so that a lane ends up with
// four consecutive output columns of one output row (an 8-byte bf16 store).
#pragma once
#include <type_traits>
#include "common.h"

namespace ditron {

// 16 zero bytes in global memory: lanes whose K-chunk lies beyond the contraction length
// stage these instead (the direct-to-LDS load has no per-lane zero fill).
__device__ const u32x4_t kZeroChunk = {0u, 0u, 0u, 0u};

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, BK = 64, NSTAGE = 2;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NWAVES = WAVES_M * WAVES_N, THREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int KS = BK / 16;                    // MFMA steps per K tile
  static constexpr int ROW_BYTES = 128;                 // BK bf16 = one cache line per row per K tile
  static constexpr int ROWS_PER_LOAD = 8;               // rows written by one wave-wide 1 KiB load
  // the four waves of the first group stage the A rows, the four of the second group the B rows
  static constexpr int A_LOADS = BM / ROWS_PER_LOAD / 4;
  static constexpr int B_LOADS = BN / ROWS_PER_LOAD / 4;
  static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
  static constexpr int kSchedule = 0;   // ping-pong
  static_assert(NWAVES == 8, "two groups of four waves (one wave of each group per SIMD)");
  static_assert(BM == BN, "both groups issue the same number of loads");
  static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile must be 32-aligned");
  static_assert(A_LOADS <= 15, "wait counts are 4-bit immediates");
};

// Chunk swizzle for 128-byte LDS rows (eight 16-byte chunks): chunk c of row r is stored at
// chunk position c ^ swz128(r).  Makes 128-bit reads of 8 or of 16 consecutive rows at one
// logical chunk hit distinct banks; invariant under adding a multiple of 16 rows.
__device__ __forceinline__ int swz128(int r) { return (r & 7) ^ ((r >> 3) & 1); }

// The explicit waits are pinned in place: the scheduler must not move matrix instructions
// behind them (a wave blocked in a wait issues nothing).
__device__ __forceinline__ void wait_vmcnt0() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __builtin_amdgcn_sched_barrier(0);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 15, "vmcnt immediate");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70 | N);
  __builtin_amdgcn_sched_barrier(0);
}
__device__ __forceinline__ void wait_lgkmcnt0() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_sched_barrier(0);
}

// Work-group barrier that leaves outstanding global loads in flight (the plain
// __syncthreads() drains them).  The empty asm statements stop the compiler from moving
// memory accesses across it; sched_barrier keeps the instruction scheduler from moving
// anything else (the phases of the two wave groups must not be blended).
__device__ __forceinline__ void barrier_no_drain() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");
}

// Direct global -> LDS staging of one operand's rows of a K tile by a group of four waves.
// A wave-wide load writes 1 KiB = 8 rows x 128 B; the LDS side of that write is fixed
// (lane i writes bytes [16 i, 16 i + 16)), so the row swizzle is applied on the global side:
// the lane that fills chunk position p of row r fetches chunk p ^ swz128(r).
template <int NLOADS>
struct HalfLoader {
  const char* base;           // operand base address (uniform)
  uint32_t off[NLOADS];       // this lane's byte offset from `base` for K tile 0, per load instruction
  int wave4;                  // wave index inside the group

  // row(r): byte offset (from `base_`) of the start of tile-local row r, already clamped to a valid row
  template <class Row>
  __device__ __forceinline__ void init(const char* base_, Row row, int wave_in_group) {
    const int lane = threadIdx.x & 63;
    base = base_;
    wave4 = wave_in_group;
#pragma unroll
    for (int i = 0; i < NLOADS; ++i) {
      const int r = (wave_in_group * NLOADS + i) * 8 + (lane >> 3);
      const int c = (lane & 7) ^ swz128(r);
      off[i] = row(r) + (uint32_t)(c * 16);
    }
  }

  // Start this group's loads of K tile `kt` into the operand area at `dst` of an LDS stage.
  template <bool PARTIAL>
  __device__ __forceinline__ void issue(char* dst, int kt, int K) const {
    const int lane = threadIdx.x & 63;
    const char* tile_base = base + (size_t)kt * 128;
    // keep the uniform part of the address in scalar registers: the loads then take the form
    // "scalar base + 32-bit lane offset" and no 64-bit per-lane addresses have to be kept alive
    asm volatile("" : "+s"(tile_base));
#pragma unroll
    for (int i = 0; i < NLOADS; ++i) {
      const char* src = tile_base + off[i];
      if (PARTIAL) {
        const int r = (wave4 * NLOADS + i) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz128(r);
        if (kt * 64 + c * 8 >= K) src = (const char*)&kZeroChunk;
      }
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(dst + (wave4 * NLOADS + i) * 1024), 16, 0, 0);
    }
  }
};

// All operand fragments of one K tile for the calling wave (KS steps of 16).
template <class T>
struct Frags {
  bf16x8_t a[T::KS][T::MI];
  bf16x8_t b[T::KS][T::NI];
};

template <class T>
__device__ __forceinline__ void load_frags(Frags<T>& f, const char* stage, int a_off, int b_off, int sw, int lh) {
#pragma unroll
  for (int ks = 0; ks < T::KS; ++ks) {
    const int off = ((ks * 2 + lh) ^ sw) * 16;
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni) f.b[ks][ni] = *(const bf16x8_t*)(stage + b_off + ni * 32 * T::ROW_BYTES + off);
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi) f.a[ks][mi] = *(const bf16x8_t*)(stage + a_off + mi * 32 * T::ROW_BYTES + off);
  }
}

// acc[ni][mi] is the 32x32 block whose instruction rows are B rows wn*WTN + ni*32.. and whose
// instruction columns are A rows wm*WTM + mi*32...
template <class T>
__device__ __forceinline__ void mma_tile(f32x16_t (&acc)[T::NI][T::MI], const Frags<T>& f) {
#pragma unroll
  for (int ks = 0; ks < T::KS; ++ks)
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < T::MI; ++mi)
        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ks][ni], f.a[ks][mi], acc[ni][mi], 0, 0, 0);
}

// Which WTM x WTN sub-tile of the output tile a wave owns.  Waves w and w+4 (same SIMD, one
// of each group) get neighbouring sub-tiles.
template <class T>
__device__ __forceinline__ void wave_subtile(int& wm, int& wn) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wt = T::NWAVES == 8 ? (wave & 3) * 2 + (wave >> 2) : wave;
  wm = wt / T::WAVES_N;
  wn = wt % T::WAVES_N;
}

// ------------------------------------------------------------------ 4-wave tile
// 256 x 256 output tile computed by four waves, one per SIMD, each owning 128 x 128 (256
// accumulator registers).  Compared with the 8-wave tile every fragment read from LDS feeds
// twice as many MFMAs, and operands are staged global -> registers -> LDS (plain loads of
// full 128-byte lines stream from L2 faster than the direct-to-LDS form).  LDS holds two
// stages of one 64-deep K tile each, rows of 128 bytes with the same chunk swizzle as the
// 8-wave tile (measured free of bank conflicts for both the fragment reads and the stores).
struct GemmTile4W {
  static constexpr int BM = 256, BN = 256, BK = 64, NSTAGE = 2;
  static constexpr int WAVES_M = 2, WAVES_N = 2, NWAVES = 4, THREADS = 256;
  static constexpr int WTM = 128, WTN = 128, MI = 4, NI = 4;
  static constexpr int kSchedule = 1;
  static constexpr int ROW_BYTES = 128;
  static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
  static constexpr int ROWS_PER_PASS = THREADS / 8;           // 32 rows per pass of 16-byte loads
  static constexpr int A_LOADS = BM / ROWS_PER_PASS, B_LOADS = BN / ROWS_PER_PASS, LOADS = A_LOADS + B_LOADS;
};

struct Frags4W {
  bf16x8_t a[4];
  bf16x8_t b[4];
};

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Fragment J of step KS (0..3) of the K tile staged at `st`.  koff[KS] is the lane's swizzled
// chunk offset for that step.  The order (b0, a0..a3, b1..b3) is the order in which mma_pair
// consumes them.
template <int KS, int J>
__device__ __forceinline__ void read_one(Frags4W& f, const char* st, int a_off, int b_off, const int (&koff)[4]) {
  const int off = koff[KS];
  if constexpr (J == 0) f.b[0] = *(const bf16x8_t*)(st + b_off + off);
  else if constexpr (J <= 4) f.a[J - 1] = *(const bf16x8_t*)(st + a_off + (J - 1) * 32 * 128 + off);
  else f.b[J - 4] = *(const bf16x8_t*)(st + b_off + (J - 4) * 32 * 128 + off);
}

template <int P>
__device__ __forceinline__ void mma_pair(f32x16_t (&acc)[4][4], const Frags4W& f) {
  constexpr int ni = P / 2, mi = (P % 2) * 2;
  acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi], acc[ni][mi], 0, 0, 0);
  acc[ni][mi + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ni], f.a[mi + 1], acc[ni][mi + 1], 0, 0, 0);
}

struct Stager4W {
  typedef GemmTile4W T;
  static constexpr int kOutOfRange = 0x7ffffff0;
  __amdgpu_buffer_rsrc_t a_rsrc, b_rsrc;
  int off[T::LOADS];
  u32x4_t reg[1][T::LOADS];
  int lds_off;    // byte offset inside an operand area of a stage, pass 0
  int kc;

  template <class ARow, class BRow>
  __device__ __forceinline__ void init(const char* a_base, ARow a_row, const char* b_base, BRow b_row) {
    const int r = threadIdx.x >> 3, c = threadIdx.x & 7;
    a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a_base, 0, kOutOfRange, 0x00020000);
    b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)b_base, 0, kOutOfRange, 0x00020000);
    kc = c * 8;
    lds_off = r * T::ROW_BYTES + ((c ^ swz128(r)) * 16);
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) off[i] = (int)(a_row(r + i * T::ROWS_PER_PASS) + (uint32_t)(c * 16));
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i)
      off[T::A_LOADS + i] = (int)(b_row(r + i * T::ROWS_PER_PASS) + (uint32_t)(c * 16));
  }

  // `kt` must be a valid K tile; a chunk past K reads as zero (lane offset pushed out of range)
  template <int SET, int I>
  __device__ __forceinline__ void fetch_one(int kt, int K) {
    const bool dead = kt * 64 + kc >= K;
    const int v = dead ? kOutOfRange : off[I];
    reg[SET][I] = __builtin_amdgcn_raw_buffer_load_b128(I < T::A_LOADS ? a_rsrc : b_rsrc, v, kt * 128, 0);
  }
  template <int SET>
  __device__ __forceinline__ void fetch(int kt, int K) {
    static_for<0, T::LOADS>([&](auto i) { fetch_one<SET, decltype(i)::value>(kt, K); });
  }

  // `pair`: the stage that receives the K tile
  template <int SET, int I>
  __device__ __forceinline__ void commit_one(char* pair) const {
    constexpr int area = I < T::A_LOADS ? 0 : T::A_BYTES;
    constexpr int pass = I < T::A_LOADS ? I : I - T::A_LOADS;
    *(u32x4_t*)(pair + area + lds_off + pass * T::ROWS_PER_PASS * T::ROW_BYTES) = reg[SET][I];
  }
  template <int SET>
  __device__ __forceinline__ void commit(char* pair) const {
    static_for<0, T::LOADS>([&](auto i) { commit_one<SET, decltype(i)::value>(pair); });
  }
};

// One barrier per 64-deep K tile.  A single wave per SIMD has to keep the matrix pipe fed
// while it also issues every memory instruction, so the loop body is written as 32 slots of
// two MFMAs plus at most three memory instructions, each slot fenced so that the compiler
// keeps the interleaving:
//   steps ks0, ks1 of tile kt : fragments of the next step; LDS stores of tile kt+1
//   step  ks2                : fragments of ks3
//   barrier
//   step  ks3                : first fragments of tile kt+1
//   every other slot         : one global load of tile kt+2
// The body is branch-free (past the end the last tile is staged again into a free stage).
template <class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop_4w(f32x16_t (&acc)[4][4], const char* a_base, ARow a_row,
                                                 const char* b_base, BRow b_row, int K, char* lds) {
  typedef GemmTile4W T;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 31, lh = lane >> 5;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  const int b_off = T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + lh) ^ swz128(lr)) * 16;
#pragma unroll
  for (int ni = 0; ni < 4; ++ni)
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;

  const int kt_all = (K + 63) / 64;
  const int kt_last = kt_all - 1;
  Stager4W st;
  st.init(a_base, a_row, b_base, b_row);
  st.template fetch<0>(0, K);
  st.template commit<0>(lds);
  st.template fetch<0>(min(1, kt_last), K);
  __syncthreads();

  Frags4W f0, f1;
  static_for<0, 8>([&](auto j) { read_one<0, decltype(j)::value>(f0, lds, a_off, b_off, koff); });
  for (int kt = 0; kt < kt_all; ++kt) {
    constexpr int SET = 0;
    const char* cur = lds + (kt & 1) * T::STAGE_BYTES;
    char* nxt = lds + ((kt + 1) & 1) * T::STAGE_BYTES;
    const int kf = min(kt + 2, kt_last);
    static_for<0, 32>([&](auto sl) {
      constexpr int S = decltype(sl)::value, PART = S / 8, J = S % 8;
      if constexpr (S == 24) {
        wait_lgkmcnt0();   // own LDS stores of tile kt+1 are done and every read of tile kt has returned
        barrier_no_drain();
      }
      mma_pair<J>(acc, (PART & 1) ? f1 : f0);
      if constexpr (PART == 0) read_one<1, J>(f1, cur, a_off, b_off, koff);
      if constexpr (PART == 1) read_one<2, J>(f0, cur, a_off, b_off, koff);
      if constexpr (PART == 2 && J < 4) {   // early, so that the wait before the barrier finds them done
        read_one<3, 2 * J>(f1, cur, a_off, b_off, koff);
        read_one<3, 2 * J + 1>(f1, cur, a_off, b_off, koff);
      }
      if constexpr (PART == 3 && J < 4) {
        read_one<0, 2 * J>(f0, nxt, a_off, b_off, koff);
        read_one<0, 2 * J + 1>(f0, nxt, a_off, b_off, koff);
      }
      // register i goes to LDS in slot i and is refilled (tile kt+2) in slot 2i+1:
      // the loads are spread over the whole iteration, since a burst would saturate the
      // address unit and stall the wave
      if constexpr (S < 16) st.template commit_one<SET, S>(nxt);
      if constexpr (S % 2 == 1) st.template fetch_one<SET, S / 2>(kf, K);
      __builtin_amdgcn_sched_barrier(0);
    });
  }
}

template <class T, class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop(f32x16_t (&acc)[T::NI][T::MI], const char* a_base, ARow a_row,
                                              const char* b_base, BRow b_row, int K, char* lds) {
  if constexpr (T::kSchedule == 1) {
    gemm_mainloop_4w(acc, a_base, a_row, b_base, b_row, K, lds);
    return;
  } else {
  static_assert(T::NSTAGE == 2 && T::BK == 64, "pipeline below is written for 2 stages of 64");
  constexpr int NL = T::A_LOADS;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int group = wave >> 2;                 // 0: waves 0-3, 1: waves 4-7
  int wm, wn;
  wave_subtile<T>(wm, wn);
  const int lr = lane & 31, lh = lane >> 5;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  const int b_off = T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  const int sw = swz128(lr);
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;

  const int kt_full = K / T::BK;
  const int kt_all = (K + T::BK - 1) / T::BK;
  HalfLoader<NL> ld;
  if (group == 0) ld.init(a_base, a_row, wave & 3);
  else ld.init(b_base, b_row, wave & 3);
  const int half_off = group == 0 ? 0 : T::A_BYTES;
  auto issue = [&](int kt) {
    char* dst = lds + (kt & 1) * T::STAGE_BYTES + half_off;
    if (kt < kt_full) ld.template issue<false>(dst, kt, K);
    else ld.template issue<true>(dst, kt, K);
  };

  issue(0);
  if (kt_all > 1) {
    issue(1);
    wait_vmcnt<NL>();
  } else {
    wait_vmcnt0();
  }
  barrier_no_drain();   // tile 0 is in LDS

  Frags<T> f;
  if (group == 0) {
    load_frags<T>(f, lds, a_off, b_off, sw, lh);
    for (int kt = 0; kt < kt_all; ++kt) {
      wait_lgkmcnt0();
      barrier_no_drain();                        // even phase starts: this group multiplies tile kt
      mma_tile<T>(acc, f);
      wait_vmcnt0();                             // own share of tile kt+1 has landed
      barrier_no_drain();                        // odd phase starts: the other group multiplies tile kt
      if (kt + 2 < kt_all) issue(kt + 2);        // stage kt&1 has been read by both groups
      if (kt + 1 < kt_all) load_frags<T>(f, lds + ((kt + 1) & 1) * T::STAGE_BYTES, a_off, b_off, sw, lh);
    }
  } else {
    for (int kt = 0; kt < kt_all; ++kt) {
      barrier_no_drain();                        // even phase: fetch the fragments of tile kt
      load_frags<T>(f, lds + (kt & 1) * T::STAGE_BYTES, a_off, b_off, sw, lh);
      wait_vmcnt0();                             // own share of tile kt+1 has landed
      wait_lgkmcnt0();                           // and the fragment reads are done: the stage may be refilled
      barrier_no_drain();                        // odd phase: multiply tile kt
      if (kt + 2 < kt_all) issue(kt + 2);
      mma_tile<T>(acc, f);
    }
  }
  }
}

// Store the wave's accumulators as bf16 into row-major C (leading dimension ldc elements),
// tile origin (m0, n0), bounds (M, N).  row_scale / col_scale may be null.
template <class T>
__device__ __forceinline__ void store_tile_bf16(const f32x16_t (&acc)[T::NI][T::MI], __bf16* c, size_t ldc,
                                                int m0, int n0, int M, int N, const float* row_scale,
                                                int rows_per_scale, const float* col_scale) {
  const int lane = threadIdx.x & 63;
  int wm, wn;
  wave_subtile<T>(wm, wn);
  const int lr = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi) {
    const int m = m0 + wm * T::WTM + mi * 32 + lr;
    if (m >= M) continue;
    const float rs = row_scale ? row_scale[m / rows_per_scale] : 1.f;
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * T::WTN + ni * 32 + g * 8 + lh * 4;
        if (n >= N) continue;
        float x0 = acc[ni][mi][g * 4 + 0], x1 = acc[ni][mi][g * 4 + 1];
        float x2 = acc[ni][mi][g * 4 + 2], x3 = acc[ni][mi][g * 4 + 3];
        if (row_scale || col_scale) {
          x0 *= rs * (col_scale ? col_scale[n] : 1.f);
          x1 *= rs * (col_scale && n + 1 < N ? col_scale[n + 1] : 1.f);
          x2 *= rs * (col_scale && n + 2 < N ? col_scale[n + 2] : 1.f);
          x3 *= rs * (col_scale && n + 3 < N ? col_scale[n + 3] : 1.f);
        }
        __bf16* dst = c + (size_t)m * ldc + n;
        if (n + 3 < N) {
          bf16x4_t v = {(__bf16)x0, (__bf16)x1, (__bf16)x2, (__bf16)x3};
          *(bf16x4_t*)dst = v;
        } else {
          dst[0] = (__bf16)x0;
          if (n + 1 < N) dst[1] = (__bf16)x1;
          if (n + 2 < N) dst[2] = (__bf16)x2;
        }
      }
    }
  }
}

// Epilogue of the 4-wave tile: each wave turns its 128 x 128 accumulators into bf16, parks
// them in its own 32 KiB of the (now idle) operand stages, and reads them back row by row so
// that every global store covers whole 128-byte lines (16 lanes x 16 bytes per row; written
// straight from the MFMA layout, a store instruction would scatter 8-byte pieces over 32
// rows).  Rows are 256 bytes; the 16-byte slot g of row m lives at slot g ^ (m & 15), which
// keeps both the 8-byte writes and the 16-byte reads free of bank conflicts.
__device__ __forceinline__ void store_tile_bf16_lds(const f32x16_t (&acc)[4][4], __bf16* c, size_t ldc, int m0,
                                                    int n0, int M, int N, char* lds) {
  typedef GemmTile4W T;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 31, lh = lane >> 5;
  __syncthreads();   // every wave is done reading the operand stages
  char* park = lds + wave * (T::WTM * T::WTN * 2);
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = mi * 32 + lr;
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int g = ni * 4 + q;
        bf16x4_t v = {(__bf16)acc[ni][mi][q * 4 + 0], (__bf16)acc[ni][mi][q * 4 + 1],
                      (__bf16)acc[ni][mi][q * 4 + 2], (__bf16)acc[ni][mi][q * 4 + 3]};
        *(bf16x4_t*)(park + m * 256 + ((g ^ (m & 15)) * 16) + lh * 8) = v;
      }
    }
  }
  // the reads below are the same wave's: LDS operations of one wave complete in order
  wait_lgkmcnt0();
  const int g = lane & 15;
  const int gn = n0 + wn * T::WTN + g * 8;
#pragma unroll 8
  for (int it = 0; it < T::WTM / 4; ++it) {
    const int row = it * 4 + (lane >> 4);
    const u32x4_t v = *(const u32x4_t*)(park + row * 256 + ((g ^ (row & 15)) * 16));
    const int gm = m0 + wm * T::WTM + row;
    if (gm < M && gn < N) *(u32x4_t*)(c + (size_t)gm * ldc + gn) = v;
  }
}

}  // namespace ditron
