// bf16 MFMA tile engine for gfx950: C_tile[BM,BN] (fp32) += A_tile[BM,K] . B_tile[BN,K]^T.
//
// Both operands are read as rows that are contiguous along the contraction dimension.
// A K-slice of BK=64 elements of BM + BN rows is staged in LDS as 128-byte rows whose eight
// 16-byte chunks are XOR-swizzled by the row index; the staging uses the direct
// global->LDS load (each wave writes 1 KiB = 8 consecutive rows per instruction, the
// swizzle is applied on the global-address side).  Each wave owns a WTM x WTN sub-tile and
// feeds v_mfma_f32_32x32x16_bf16 from 128-bit LDS reads.  The instruction's row operand is
// taken from the B rows and its column operand from the A rows, so that a lane ends up with
// four consecutive output columns of one output row (an 8-byte bf16 store).
#pragma once
#include "common.h"

namespace ditron {

// 16 zero bytes in global memory: lanes whose K-chunk lies beyond the contraction length
// stage these instead (the direct-to-LDS load has no per-lane zero fill).
__device__ const u32x4_t kZeroChunk = {0u, 0u, 0u, 0u};

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_, int NSTAGE_ = 2>
struct GemmTile {
  static constexpr int BM = BM_, BN = BN_, BK = 64, NSTAGE = NSTAGE_;
  static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NWAVES = WAVES_M * WAVES_N, THREADS = 64 * NWAVES;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  static constexpr int MI = WTM / 32, NI = WTN / 32;
  static constexpr int ROW_BYTES = 128;                 // BK bf16
  static constexpr int ROWS_PER_LOAD = 8;               // rows written by one wave-wide load
  static constexpr int A_LOADS = BM / ROWS_PER_LOAD / NWAVES;
  static constexpr int B_LOADS = BN / ROWS_PER_LOAD / NWAVES;
  static constexpr int LOADS = A_LOADS + B_LOADS;
  static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
  static_assert(BM % (32 * WAVES_M) == 0 && BN % (32 * WAVES_N) == 0, "wave tile must be 32-aligned");
  static_assert(BM % (ROWS_PER_LOAD * NWAVES) == 0 && BN % (ROWS_PER_LOAD * NWAVES) == 0, "load split");
};

// Chunk swizzle: the 16-byte chunk c of LDS row r is stored at chunk position c ^ swz(r).
// Conflict-free for 128-bit reads of 8 or 16 consecutive rows at one logical chunk.
__device__ __forceinline__ int swz(int r) { return (r & 7) ^ ((r >> 3) & 1); }

__device__ __forceinline__ void wait_vmcnt0() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <class T>
struct TileLoader {
  const char* ptr[T::LOADS];  // this lane's source address for K tile 0, per load instruction
  int kc[T::LOADS];           // element offset of the lane's chunk inside a K tile

  // a_row(r) / b_row(r): start of tile-local row r (already clamped to a valid row).
  template <class ARow, class BRow>
  __device__ __forceinline__ void init(ARow a_row, BRow b_row) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
      const int r = (wave * T::A_LOADS + i) * T::ROWS_PER_LOAD + (lane >> 3);
      const int c = (lane & 7) ^ swz(r);
      kc[i] = c * 8;
      ptr[i] = a_row(r) + c * 16;
    }
#pragma unroll
    for (int i = 0; i < T::B_LOADS; ++i) {
      const int r = (wave * T::B_LOADS + i) * T::ROWS_PER_LOAD + (lane >> 3);
      const int c = (lane & 7) ^ swz(r);
      kc[T::A_LOADS + i] = c * 8;
      ptr[T::A_LOADS + i] = b_row(r) + c * 16;
    }
  }

  // Start the loads of K tile `kt` into the LDS stage at `stage`.
  template <bool PARTIAL>
  __device__ __forceinline__ void issue(char* stage, int kt, int K) const {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int i = 0; i < T::LOADS; ++i) {
      const char* src = ptr[i] + (size_t)kt * T::ROW_BYTES;
      if (PARTIAL) {
        if (kt * T::BK + kc[i] >= K) src = (const char*)&kZeroChunk;
      }
      char* dst = (i < T::A_LOADS)
                      ? stage + (wave * T::A_LOADS + i) * 1024
                      : stage + T::A_BYTES + (wave * T::B_LOADS + (i - T::A_LOADS)) * 1024;
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(dst), 16, 0, 0);
    }
  }
};

// One K tile of MFMA work for the calling wave.  acc[ni][mi] is the 32x32 block whose
// instruction rows are B rows wn*WTN + ni*32.. and instruction columns A rows wm*WTM + mi*32...
template <class T>
__device__ __forceinline__ void mma_stage(f32x16_t (&acc)[T::NI][T::MI], const char* stage, int wm, int wn) {
  const int lane = threadIdx.x & 63;
  const int lr = lane & 31, lh = lane >> 5;
  const char* a_base = stage + (wm * T::WTM + lr) * T::ROW_BYTES;
  const char* b_base = stage + T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  const int sw = swz(lr);  // tile bases are multiples of 32, so the swizzle depends on lr only
#pragma unroll
  for (int ks = 0; ks < T::BK / 16; ++ks) {
    const int off = ((ks * 2 + lh) ^ sw) * 16;
    bf16x8_t af[T::MI], bfr[T::NI];
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni) bfr[ni] = *(const bf16x8_t*)(b_base + ni * 32 * T::ROW_BYTES + off);
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi) af[mi] = *(const bf16x8_t*)(a_base + mi * 32 * T::ROW_BYTES + off);
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
      for (int mi = 0; mi < T::MI; ++mi)
        acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[ni][mi], 0, 0, 0);
  }
}

// Full contraction for one output tile.  K must be a multiple of 8; the last K tile may be
// partial.  `lds` is T::LDS_BYTES of dynamic shared memory.
template <class T, class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop(f32x16_t (&acc)[T::NI][T::MI], ARow a_row, BRow b_row, int K,
                                              char* lds) {
  static_assert(T::NSTAGE == 2, "two LDS stages");
  const int wave = threadIdx.x >> 6;
  const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;

  TileLoader<T> loader;
  loader.init(a_row, b_row);
  const int kt_full = K / T::BK;
  const int kt_all = (K + T::BK - 1) / T::BK;

  if (kt_full > 0) loader.template issue<false>(lds, 0, K);
  else loader.template issue<true>(lds, 0, K);

  for (int kt = 0; kt < kt_all; ++kt) {
    wait_vmcnt0();
    __syncthreads();  // tile kt has landed for every wave; every wave has finished tile kt-1
    const int nxt = kt + 1;
    if (nxt < kt_full) loader.template issue<false>(lds + (nxt & 1) * T::STAGE_BYTES, nxt, K);
    else if (nxt < kt_all) loader.template issue<true>(lds + (nxt & 1) * T::STAGE_BYTES, nxt, K);
    mma_stage<T>(acc, lds + (kt & 1) * T::STAGE_BYTES, wm, wn);
  }
}

// Store the wave's accumulators as bf16 into row-major C (leading dimension ldc elements),
// tile origin (m0, n0), bounds (M, N).  row_scale / col_scale may be null.
template <class T>
__device__ __forceinline__ void store_tile_bf16(const f32x16_t (&acc)[T::NI][T::MI], __bf16* c, size_t ldc,
                                                int m0, int n0, int M, int N, const float* row_scale,
                                                int rows_per_scale, const float* col_scale) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave / T::WAVES_N, wn = wave % T::WAVES_N;
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

}  // namespace ditron
