// bf16 MFMA tile engine for gfx950: C_tile[BM,BN] (fp32) += A_tile[BM,K] . B_tile[BN,K]^T.
//
// Both operands are read as rows that are contiguous along the contraction dimension.  A
// K slice of 64 elements of BM + BN rows is staged in LDS as 128-byte rows (one cache line per
// row) whose eight 16-byte chunks are XOR-swizzled by the row index.  Four waves, one per SIMD,
// each own a quarter of the tile and feed v_mfma_f32_32x32x16_bf16 (or, in the X16 form of the tile,
// v_mfma_f32_16x16x32_bf16) from 128-bit LDS reads.  The
// instruction's row operand is taken from the B rows and its column operand from the A rows,
// so that a lane ends up with four consecutive output columns of one output row.
#pragma once
#include <type_traits>
#include "common.h"

namespace ditron {

// 16 zero bytes in global memory, for kernels that stage operands with the direct-to-LDS load
// (it has no per-lane zero fill): lanes whose K-chunk lies beyond the contraction length stage
// these instead.
__device__ const u32x4_t kZeroChunk = {0u, 0u, 0u, 0u};

// Chunk swizzle for 128-byte LDS rows (eight 16-byte chunks): chunk c of row r is stored at
// chunk position c ^ swz128(r).  Makes 128-bit reads of 8 or of 16 consecutive rows at one
// logical chunk hit distinct banks; invariant under adding a multiple of 16 rows.
__device__ __forceinline__ int swz128(int r) { return (r & 7) ^ ((r >> 3) & 1); }
// The same for the 16 x 16 x 32 form, whose 128-bit reads take the four chunks of a 32-deep step of 16
// consecutive rows (lane = 16 chunk + row): measured on the chip with the LDS saturated, that read takes 1.64
// times as long under swz128 as under this one (and the 32-row read above 1.64 times as long under this one).
__device__ __forceinline__ int swz128_x16(int r) { return r & 7; }

// The explicit waits are pinned in place: the scheduler must not move matrix instructions
// behind them (a wave blocked in a wait issues nothing).
__device__ __forceinline__ void wait_vmcnt0() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __builtin_amdgcn_sched_barrier(0);
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 63, "vmcnt immediate (six bits: [3:0] and [15:14])");
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
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

// ------------------------------------------------------------------ the tile
// BM x BN output tile (BM 256 or 128, BN 256, 192 or 128) computed by four waves, one per SIMD,
// each owning BM/2 x BN/2 (256 x 256: 128 x 128 per wave, 256 accumulator registers, every
// fragment read from LDS feeds four MFMAs).  Operands are staged global -> registers -> LDS, or,
// with DIRECT, global -> LDS (`buffer_load ... lds`; measured faster on 256 x 256 tiles whose
// contraction is a whole number of K tiles, slower for a ragged last K tile and on 128-row tiles,
// so the launch code picks per problem).  LDS holds two stages of one 64-deep K tile each (the
// 16 x 16 x 32 form: a ring of five half stages), rows of 128 bytes (measured free of bank
// conflicts for both the fragment reads and the staging stores).
//
// B_KN: B is stored [K, N] (N contiguous) instead of [N, K].  Its K tile is then staged as it
// lies in memory, 64 rows of BN elements with a pitch of 2 BN + 64 bytes, and the MFMA
// operand (eight consecutive k of one column per lane) is assembled by two transposing LDS
// reads (ds_read_b64_tr_b16: inside each group of 16 lanes, lane i receives element i % 4 of
// the 8-byte chunks addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4; measured).  The pitch
// makes the four rows a group touches, and the two groups that share a cycle, hit distinct banks.
//
// X16: the same tile fed to v_mfma_f32_16x16x32_bf16 (a wave's quarter is cut into 16 x 16 blocks, a fragment
// is 16 rows x 32 k: the 16-byte chunk (lane / 16) of the 32-deep step of row (lane % 16)); written for the
// direct-to-LDS staging.  The accumulator of a block is four registers instead of sixteen, so the instruction
// moves a quarter of the accumulator registers per unit of matrix work.
template <int BM_, int BN_, bool B_KN_ = false, bool DIRECT_ = false, bool X16_ = false>
struct GemmTile4W {
  static_assert((BM_ == 256 || BM_ == 128) && (BN_ == 256 || BN_ == 192 || BN_ == 128 || (X16_ && BN_ == 224)), "supported tile sides");
  static_assert(!B_KN_ || BN_ != 192, "a [K, N] row of 192 elements does not split evenly over the loading lanes");
  static_assert(!DIRECT_ || !B_KN_, "the direct-to-LDS staging is written for [N, K] operands");
  static_assert(!X16_ || DIRECT_, "the 16 x 16 x 32 loop is written for the direct-to-LDS staging");
  static_assert(!X16_ || (BN_ <= BM_ && BN_ % 32 == 0), "the 16 x 16 x 32 loop keeps A and B parts in one ring of pieces the size of the A part");
  static constexpr bool B_KN = B_KN_;
  static constexpr bool DIRECT = DIRECT_;   // operands go from global memory straight into LDS (no staging registers)
  static constexpr bool X16 = X16_;
  static constexpr int BM = BM_, BN = BN_, BK = 64, NSTAGE = 2;
  static constexpr int WAVES_M = 2, WAVES_N = 2, NWAVES = 4, THREADS = 256;
  static constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;
  static constexpr int ROW_BYTES = 128;
  static constexpr int PB = BN * 2 + 64;                      // B_KN: bytes between two k rows of the staged B tile
  static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = B_KN ? BK * PB : BN * ROW_BYTES;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  // X16: a ring of five operand pieces (the A part and the B part of a K tile are pieces of their own), all of the LDS
  static constexpr int LDS_BYTES = X16_ ? 5 * A_BYTES : NSTAGE * STAGE_BYTES;
  static constexpr int ROWS_PER_PASS = THREADS / 8;           // 32 rows per pass of 16-byte loads
  static constexpr int A_LOADS = BM / ROWS_PER_PASS, B_LOADS = BN / ROWS_PER_PASS, LOADS = A_LOADS + B_LOADS;
  // The K loop is written as slots of two MFMAs (one B fragment, two A fragments).
  static constexpr int PAIRS = MI * NI / 2;                   // slots per 16-deep step
  static constexpr int SLOTS = 4 * PAIRS;                     // slots per 64-deep K tile
  static constexpr int B_READS = B_KN ? 2 : 1;                // LDS reads per B fragment
  static constexpr int READS = MI + B_READS * NI;             // fragment reads per step
  static constexpr int HALF = (PAIRS + 1) / 2;                // slots of a step that take its reads when they must be early
  static constexpr int MB = WTM / 16, NB = WTN / 16;          // X16: 16 x 16 blocks of a wave's quarter
  // the accumulators of one wave: [column block][row block]
  typedef f32x16_t Acc32[NI][MI];
  typedef f32x4_t Acc16[NB][MB];
  typedef std::conditional_t<X16_, Acc16, Acc32> Acc;
};

template <class T>
struct Frags4W {
  bf16x8_t a[T::MI];
  bf16x4_t b[T::NI][2];   // low and high four k of the fragment ([N, K] storage fills both with one read)
};

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// B fragment NI_ of step KS: READ 0 (and, for [K, N] storage, READ 1 for the upper four k).
// b_off is the lane's base inside the stage: for [N, K] storage the row of its column, for
// [K, N] storage the chunk it addresses in the transposing read.
template <class T, int KS, int NI_, int READ>
__device__ __forceinline__ void read_b(Frags4W<T>& f, const char* st, int b_off, const int (&koff)[4]) {
  if constexpr (T::B_KN) {
    const char* src = st + b_off + NI_ * 64 + (KS * 16 + READ * 4) * T::PB;
    const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)DITRON_LDS(src));
    f.b[NI_][READ] = __builtin_bit_cast(bf16x4_t, v);
  } else {
    const bf16x8_t v = *(const bf16x8_t*)(st + b_off + NI_ * 32 * 128 + koff[KS]);
    f.b[NI_][0] = __builtin_shufflevector(v, v, 0, 1, 2, 3);
    f.b[NI_][1] = __builtin_shufflevector(v, v, 4, 5, 6, 7);
  }
}

// Fragment read J of step KS (0..3) of the K tile staged at `st`.  koff[KS] is the lane's
// swizzled chunk offset for that step.  The order (b0, a0..a[MI-1], b1..b[NI-1]) is the order
// in which mma_pair consumes them.
template <class T, int KS, int J>
__device__ __forceinline__ void read_one(Frags4W<T>& f, const char* st, int a_off, int b_off, const int (&koff)[4]) {
  constexpr int BR = T::B_READS;
  if constexpr (J < BR) read_b<T, KS, 0, J>(f, st, b_off, koff);
  else if constexpr (J < BR + T::MI) f.a[J - BR] = *(const bf16x8_t*)(st + a_off + (J - BR) * 32 * 128 + koff[KS]);
  else read_b<T, KS, 1 + (J - BR - T::MI) / BR, (J - BR - T::MI) % BR>(f, st, b_off, koff);
}
// reads [LO, HI) of a step
template <class T, int KS, int LO, int HI>
__device__ __forceinline__ void read_range(Frags4W<T>& f, const char* st, int a_off, int b_off, const int (&koff)[4]) {
  static_for<LO, HI>([&](auto j) { read_one<T, KS, decltype(j)::value>(f, st, a_off, b_off, koff); });
}

template <class T, int P>
__device__ __forceinline__ void mma_pair(typename T::Acc32& acc, const Frags4W<T>& f) {
  constexpr int ni = P / (T::MI / 2), mi = (P % (T::MI / 2)) * 2;
  const bf16x8_t b = __builtin_shufflevector(f.b[ni][0], f.b[ni][1], 0, 1, 2, 3, 4, 5, 6, 7);
  acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, f.a[mi], acc[ni][mi], 0, 0, 0);
  acc[ni][mi + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, f.a[mi + 1], acc[ni][mi + 1], 0, 0, 0);
}

// Where the columns of a B stored [K, N] are: the mainloop's `b_row` argument for B_KN tiles.
struct BColumns {
  uint32_t ld_bytes;   // bytes between two k rows (2 N)
  int n0, n;           // first column of the tile, number of columns of B
};

template <class T>
struct Stager4W {
  static constexpr int kOutOfRange = 0x7ffffff0;
  static constexpr int KN_LANES = T::BN / 8;              // B_KN: lanes that cover one k row of the tile
  static constexpr int KN_ROWS = T::THREADS / KN_LANES;   // B_KN: k rows per pass
  static constexpr bool kDirect = T::DIRECT;
  __amdgpu_buffer_rsrc_t a_rsrc, b_rsrc;
  int off[T::LOADS];
  u32x4_t reg[T::LOADS];
  int lds_off;    // byte offset inside an operand area of a stage, pass 0
  int kc;
  int kn_row, kn_lds_off, kn_tile_bytes;   // B_KN: the lane's k row in pass 0, its LDS offset, bytes per K tile of B
  int wave_lds;   // direct-to-LDS form: where the wave's 8 rows of a pass start

  template <class ARow, class BRow>
  __device__ __forceinline__ void init(const char* a_base, ARow a_row, const char* b_base, BRow b_row) {
    init(a_base, a_row, b_base, b_row, (int)threadIdx.x);
  }
  // tid: the thread's index among the T::THREADS threads that stage (the whole work-group, or its loading waves)
  template <class ARow, class BRow>
  __device__ __forceinline__ void init(const char* a_base, ARow a_row, const char* b_base, BRow b_row, int tid) {
    const int r = tid >> 3;
    // direct-to-LDS form: the lane's LDS position is chunk (lane & 7) of its row, which holds global chunk c
    const int c = kDirect ? ((tid & 7) ^ (T::X16 ? swz128_x16(r) : swz128(r))) : (tid & 7);
    wave_lds = __builtin_amdgcn_readfirstlane(tid >> 6) * 1024;
    a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a_base, 0, kOutOfRange, 0x00020000);
    b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)b_base, 0, kOutOfRange, 0x00020000);
    kc = c * 8;
    lds_off = r * T::ROW_BYTES + ((c ^ swz128(r)) * 16);
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) off[i] = (int)(a_row(r + i * T::ROWS_PER_PASS) + (uint32_t)(c * 16));
    if constexpr (T::B_KN) {
      // lane (k row, group of 8 columns): 16 bytes = 8 columns of one k; a wave covers whole rows of the tile
      kn_row = tid / KN_LANES;
      const int n8 = tid % KN_LANES;
      const int col = b_row.n0 + n8 * 8;
      kn_lds_off = kn_row * T::PB + n8 * 16;
      kn_tile_bytes = (int)(b_row.ld_bytes * 64u);
#pragma unroll
      for (int i = 0; i < T::B_LOADS; ++i)
        off[T::A_LOADS + i] = col < b_row.n ? (int)((uint32_t)(kn_row + i * KN_ROWS) * b_row.ld_bytes + (uint32_t)col * 2u)
                                            : kOutOfRange;   // columns past N read as zero
    } else {
#pragma unroll
      for (int i = 0; i < T::B_LOADS; ++i)
        off[T::A_LOADS + i] = (int)(b_row(r + i * T::ROWS_PER_PASS) + (uint32_t)(c * 16));
    }
  }

  // `kt` must be a valid K tile; a chunk past K reads as zero (lane offset pushed out of range)
  template <int I>
  __device__ __forceinline__ u32x4_t load_one(int kt, int K) const {
    if constexpr (T::B_KN && I >= T::A_LOADS) {
      const bool dead = kt * 64 + kn_row + (I - T::A_LOADS) * KN_ROWS >= K;
      return __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, dead ? kOutOfRange : off[I], kt * kn_tile_bytes, 0);
    } else {
      const bool dead = kt * 64 + kc >= K;
      const int v = dead ? kOutOfRange : off[I];
      return __builtin_amdgcn_raw_buffer_load_b128(I < T::A_LOADS ? a_rsrc : b_rsrc, v, kt * 128, 0);
    }
  }
  // Direct-to-LDS form of load I ([N, K] operands): the wave's 64 lanes fill 8 rows x 128 bytes that are
  // contiguous in the stage (lane l lands at byte 16 l), so the swizzle is applied on the global side: `off`
  // was built for the chunk that belongs at the lane's LDS position.  A chunk past K is pushed out of the
  // buffer's range, for which zeros are written.
  template <int I, bool WHOLE = false>
  __device__ __forceinline__ void issue_one(int kt, int K, char* stage) const {
    constexpr int area = I < T::A_LOADS ? 0 : T::A_BYTES;
    constexpr int pass = I < T::A_LOADS ? I : I - T::A_LOADS;
    const bool dead = !WHOLE && kt * 64 + kc >= K;   // WHOLE: K is a whole number of K tiles, no chunk lies past it
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass does not know this builtin
    __builtin_amdgcn_raw_ptr_buffer_load_lds(I < T::A_LOADS ? a_rsrc : b_rsrc,
                                             DITRON_LDS(stage + area + pass * T::ROWS_PER_PASS * T::ROW_BYTES + wave_lds), 16,
                                             dead ? kOutOfRange : off[I], kt * 128, 0, 0);
#else
    (void)dead; (void)stage;
#endif
  }
  template <int LO, int HI>
  __device__ __forceinline__ void issue_range(int kt, int K, char* stage) const {
    static_for<LO, HI>([&](auto i) { issue_one<decltype(i)::value>(kt, K, stage); });
  }
  template <int I>
  __device__ __forceinline__ void fetch_one(int kt, int K) { reg[I] = load_one<I>(kt, K); }
  template <int LO, int HI>
  __device__ __forceinline__ void fetch_range(int kt, int K) {
    static_for<LO, HI>([&](auto i) { fetch_one<decltype(i)::value>(kt, K); });
  }

  // `stage`: the stage that receives the K tile
  template <int I>
  __device__ __forceinline__ void commit_one(char* stage) const {
    constexpr int area = I < T::A_LOADS ? 0 : T::A_BYTES;
    constexpr int pass = I < T::A_LOADS ? I : I - T::A_LOADS;
    if constexpr (T::B_KN && I >= T::A_LOADS) *(u32x4_t*)(stage + area + kn_lds_off + pass * KN_ROWS * T::PB) = reg[I];
    else *(u32x4_t*)(stage + area + lds_off + pass * T::ROWS_PER_PASS * T::ROW_BYTES) = reg[I];
  }
  template <int LO, int HI>
  __device__ __forceinline__ void commit_range(char* stage) const {
    static_for<LO, HI>([&](auto i) { commit_one<decltype(i)::value>(stage); });
  }
};

// ------------------------------------------------------------------ 16 x 16 x 32 form
template <class T>
struct Frags16 {
  bf16x8_t a[T::MB];
  bf16x8_t b[T::NB];
};

// Fragment read J of the 32-deep step KS (0 or 1) of the K tile whose A part is staged at `pa` and whose B part
// at `pb`, in the order the slots below consume them: b0, a0 .. a[MB-1], b1 .. b[NB-1].  koff[KS]: the lane's
// swizzled chunk offset.
template <class T, int KS, int J>
__device__ __forceinline__ void read_one16(Frags16<T>& f, const char* pa, const char* pb, int a_off, int b_off,
                                            const int (&koff)[2]) {
  if constexpr (J == 0) f.b[0] = *(const bf16x8_t*)(pb + b_off + koff[KS]);
  else if constexpr (J <= T::MB) f.a[J - 1] = *(const bf16x8_t*)(pa + a_off + (J - 1) * 16 * 128 + koff[KS]);
  else f.b[J - T::MB] = *(const bf16x8_t*)(pb + b_off + (J - T::MB) * 16 * 128 + koff[KS]);
}

// MFMA I (0..3) of slot S of a step: column block S / (MB / 4), row block 4 (S % (MB / 4)) + I.
template <class T, int S, int I>
__device__ __forceinline__ void mma_one16(typename T::Acc16& acc, const Frags16<T>& f) {
  constexpr int nb = S / (T::MB / 4), mb = (S % (T::MB / 4)) * 4 + I;
  acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.b[nb], f.a[mb], acc[nb][mb], 0, 0, 0);
}

// The `n` loads of a step are spread evenly over its `slots` slots: load i goes into slot i * slots / n.  Which load
// (or none, -1) belongs to slot s.
constexpr int load_in_slot(int s, int n, int slots) {
  for (int i = 0; i < n; ++i)
    if (i * slots / n == s) return i;
  return -1;
}

// K loop of the 16 x 16 x 32 form, operands loaded straight into LDS.  WHOLE: K is a whole number of 64-deep K
// tiles and the loads carry no range test; otherwise the chunks of the last K tile that lie past K are written
// as zeros (their offsets are pushed out of the buffer's range).  A K tile is two 32-deep steps of MB x NB MFMAs each, written as slots of
// four MFMAs plus one fragment read and at most one load.  All fragments of a step are read during the step
// before it, so a K tile's operands are no longer read once its second step starts: the barrier sits between
// the two steps.  LDS is a ring of five pieces of 32 KiB; the A part of K tile j lives in piece 2j mod 5 and
// its B part in piece (2j + 1) mod 5, so two and a half K tiles are resident:
//   step 0 of tile kt : fragment reads of step 1; loads of A(kt+2) into the piece idle since the last barrier
//   barrier           : every wave's part of tile kt+1 has landed, nobody reads tile kt any more
//   step 1 of tile kt : fragment reads of step 0 of tile kt+1; loads of B(kt+2) into the piece of A(kt)
// The loads go out one per two slots over the whole K tile and have one to three steps to land (with two
// whole-tile stages all of them went out during step 1 and had one to two: at operands that are not in the
// caches, cfg 2 and cfg 3 shapes beside the vendor GEMM, the ring takes 8-10 % less time; with operands that
// are, the same).
// An MFMA of this form holds the matrix pipe for 16 cycles and the wave is alone on its SIMD, so whatever is
// issued between two MFMAs has to fit into the 12 cycles the first one leaves: the read and the load of a slot
// go behind different MFMAs, each MFMA fenced so that the compiler keeps them there (measured: with both behind
// the slot's last MFMA the loads cost ~300 and the reads ~150 cycles of a K tile's 2048; spread like this the
// cfg 2 GEMM takes 4 % less time).
// On entry the LDS must be idle; on exit no load is in flight.
template <class T, bool WHOLE, class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop_x16(typename T::Acc16& acc, const char* a_base, ARow a_row,
                                                     const char* b_base, BRow b_row, int K, char* lds) {
  constexpr int MB = T::MB, NB = T::NB, READS = MB + NB, AL = T::A_LOADS, BL = T::B_LOADS;
  constexpr int SLOTS = MB * NB / 4;   // per step
  constexpr int PIECE = T::A_BYTES;
  static_assert(MB % 4 == 0 && READS <= 2 * SLOTS && AL <= SLOTS && BL <= SLOTS && T::B_BYTES <= T::A_BYTES,
                "at most two reads and one load per slot; a B part fits in a piece");
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 15, lq = lane >> 4;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  const int b_off = (wn * T::WTN + lr) * T::ROW_BYTES;
  int koff[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) koff[ks] = ((ks * 4 + lq) ^ swz128_x16(lr)) * 16;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[nb][mb][v] = 0.f;

  const int kt_all = (K + 63) / 64;
  const int kt_last = kt_all - 1;
  Stager4W<T> st;
  st.init(a_base, a_row, b_base, b_row);
  auto wrap = [](int x) { return x >= 5 ? x - 5 : x; };
  // load I of K tile kt into the piece at `piece` (the stager puts B loads T::A_BYTES behind the address it is given)
  auto load_a = [&](auto i, int kt, char* piece) { st.template issue_one<decltype(i)::value, WHOLE>(kt, K, piece); };
  auto load_b = [&](auto i, int kt, char* piece) { st.template issue_one<AL + decltype(i)::value, WHOLE>(kt, K, piece - T::A_BYTES); };
  static_for<0, AL>([&](auto i) { load_a(i, 0, lds); });
  static_for<0, BL>([&](auto i) { load_b(i, 0, lds + PIECE); });
  static_for<0, AL>([&](auto i) { load_a(i, min(1, kt_last), lds + 2 * PIECE); });
  static_for<0, BL>([&](auto i) { load_b(i, min(1, kt_last), lds + 3 * PIECE); });
  wait_vmcnt<AL + BL>();
  barrier_no_drain();
  Frags16<T> f0, f1;
  static_for<0, READS>([&](auto j) { read_one16<T, 0, decltype(j)::value>(f0, lds, lds + PIECE, a_off, b_off, koff); });
  int ia = 0;   // piece of A(kt)
  for (int kt = 0; kt < kt_all; ++kt) {
    const char* cur_a = lds + ia * PIECE;
    const char* cur_b = lds + wrap(ia + 1) * PIECE;
    const char* nxt_a = lds + wrap(ia + 2) * PIECE;
    const char* nxt_b = lds + wrap(ia + 3) * PIECE;
    char* free_a = lds + wrap(ia + 4) * PIECE;   // held B(kt-1): nobody has read it since the last barrier
    char* free_b = lds + ia * PIECE;             // A(kt): free after this iteration's barrier
    const int kf = min(kt + 2, kt_last);   // past the end the last K tile is requested again, into pieces nobody reads
    static_for<0, SLOTS>([&](auto sl) {
      constexpr int S = decltype(sl)::value;
      mma_one16<T, S, 0>(acc, f0);
      if constexpr (S < READS) read_one16<T, 1, S>(f1, cur_a, cur_b, a_off, b_off, koff);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 1>(acc, f0);
      if constexpr (SLOTS + S < READS) read_one16<T, 1, SLOTS + S>(f1, cur_a, cur_b, a_off, b_off, koff);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 2>(acc, f0);
      if constexpr (load_in_slot(S, AL, SLOTS) >= 0) load_a(std::integral_constant<int, load_in_slot(S, AL, SLOTS)>{}, kf, free_a);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 3>(acc, f0);
      __builtin_amdgcn_sched_barrier(0);
    });
    wait_vmcnt<AL>();   // this wave's part of tile kt+1 has landed (loads return in order); A(kt+2) may be in flight
    wait_lgkmcnt0();    // every read of tile kt has returned
    barrier_no_drain();
    static_for<0, SLOTS>([&](auto sl) {
      constexpr int S = decltype(sl)::value;
      mma_one16<T, S, 0>(acc, f1);
      if constexpr (S < READS) read_one16<T, 0, S>(f0, nxt_a, nxt_b, a_off, b_off, koff);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 1>(acc, f1);
      if constexpr (SLOTS + S < READS) read_one16<T, 0, SLOTS + S>(f0, nxt_a, nxt_b, a_off, b_off, koff);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 2>(acc, f1);
      if constexpr (load_in_slot(S, BL, SLOTS) >= 0) load_b(std::integral_constant<int, load_in_slot(S, BL, SLOTS)>{}, kf, free_b);
      __builtin_amdgcn_sched_barrier(0);
      mma_one16<T, S, 3>(acc, f1);
      __builtin_amdgcn_sched_barrier(0);
    });
    ia = wrap(ia + 2);
  }
  wait_vmcnt0();   // the last iteration's requests (the last K tile once more) are not left in flight
}

// One barrier per 64-deep K tile.  A single wave per SIMD has to keep the matrix pipe fed
// while it also issues every memory instruction, so the loop body is written as slots of two
// MFMAs plus a few memory instructions, each slot fenced so that the compiler keeps the
// interleaving (four 16-deep steps ks0..ks3 of PAIRS slots each):
//   steps ks0, ks1 of tile kt : fragments of the next step; LDS stores of tile kt+1
//   step  ks2                : fragments of ks3 (in its first half)
//   barrier
//   step  ks3                : first fragments of tile kt+1 (in its first half)
//   every other slot         : global loads of tile kt+2, each after the LDS store that frees
//                               its register
// The body is branch-free (past the end the last tile is staged again into a free stage).
// On entry the LDS stages must be idle (every wave of the work-group past its last access to them): the
// direct-to-LDS staging starts writing them with its first instruction.  On exit none of the wave's loads
// is in flight; other waves may still be reading fragments, so a barrier precedes any reuse of the stages.
template <class T, class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop(typename T::Acc& acc, const char* a_base, ARow a_row,
                                                 const char* b_base, BRow b_row, int K, char* lds) {
  if constexpr (T::X16) {
    // two copies of the loop: the per-load range test of a ragged last K tile costs the others 0.8 %
    if (K % 64 == 0) gemm_mainloop_x16<T, true>(acc, a_base, a_row, b_base, b_row, K, lds);
    else gemm_mainloop_x16<T, false>(acc, a_base, a_row, b_base, b_row, K, lds);
    return;
  } else {
  constexpr int PAIRS = T::PAIRS, SLOTS = T::SLOTS, READS = T::READS, LOADS = T::LOADS;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 31, lh = lane >> 5;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  // [N, K] storage: the row of the lane's column.  [K, N] storage: the 8-byte chunk the lane
  // addresses in the transposing read: inside its group of 16 lanes, lane r points at k row r/4,
  // columns 4 (r % 4) .. +3; the group serves 16 columns, the two halves of the wave 8 k each.
  const int b_off = T::B_KN ? T::A_BYTES + (((lane & 15) >> 2) + lh * 8) * T::PB +
                                  (wn * T::WTN + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2
                            : T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + lh) ^ swz128(lr)) * 16;
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;

  const int kt_all = (K + 63) / 64;
  const int kt_last = kt_all - 1;
  Stager4W<T> st;
  st.init(a_base, a_row, b_base, b_row);
  if constexpr (Stager4W<T>::kDirect) {
    // Operands go from global memory straight into the LDS stages.  K tiles 0 and 1 are requested together;
    // inside the loop the loads of a K tile are issued over the 2 PAIRS slots that follow the barrier which
    // frees its stage (the last step of iteration kt: tile kt+2 into the stage of tile kt; the first step of
    // the next iteration: the rest of that tile), and have to be there at the next barrier.
    st.template issue_range<0, LOADS>(0, K, lds);
    st.template issue_range<0, LOADS>(min(1, kt_last), K, lds + T::STAGE_BYTES);
    wait_vmcnt<LOADS>();
    barrier_no_drain();
    Frags4W<T> f0, f1;
    read_range<T, 0, 0, READS>(f0, lds, a_off, b_off, koff);
    for (int kt = 0; kt < kt_all; ++kt) {
      char* cur = lds + (kt & 1) * T::STAGE_BYTES;
      char* nxt = lds + ((kt + 1) & 1) * T::STAGE_BYTES;
      const int kf = min(kt + 2, kt_last), kg = min(kt + 1, kt_last);
      static_for<0, SLOTS>([&](auto sl) {
        constexpr int S = decltype(sl)::value, PART = S / PAIRS, J = S % PAIRS;
        if constexpr (S == 3 * PAIRS) {
          wait_vmcnt0();     // this wave's part of tile kt+1 has landed
          wait_lgkmcnt0();   // every read of tile kt has returned
          barrier_no_drain();
        }
        mma_pair<T, J>(acc, (PART & 1) ? f1 : f0);
        if constexpr (PART == 0) read_range<T, 1, J * READS / PAIRS, (J + 1) * READS / PAIRS>(f1, cur, a_off, b_off, koff);
        if constexpr (PART == 1) read_range<T, 2, J * READS / PAIRS, (J + 1) * READS / PAIRS>(f0, cur, a_off, b_off, koff);
        if constexpr (PART == 2 && J < T::HALF)
          read_range<T, 3, J * READS / T::HALF, (J + 1) * READS / T::HALF>(f1, cur, a_off, b_off, koff);
        if constexpr (PART == 3 && J < T::HALF)
          read_range<T, 0, J * READS / T::HALF, (J + 1) * READS / T::HALF>(f0, nxt, a_off, b_off, koff);
        constexpr int W = S >= 3 * PAIRS ? S - 3 * PAIRS : S + PAIRS;   // position in the issue window
        if constexpr (W < 2 * PAIRS) {
          constexpr int LO = W * LOADS / (2 * PAIRS), HI = (W + 1) * LOADS / (2 * PAIRS);
          if constexpr (S >= 3 * PAIRS) st.template issue_range<LO, HI>(kf, K, cur);
          else st.template issue_range<LO, HI>(kg, K, nxt);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    wait_vmcnt0();   // the last iteration's requests (the last K tile once more) are not left in flight
    return;
  }
  // the first two K tiles are requested together (the second into registers that are free until the
  // loop starts), so the tile pays for one cold round trip to memory, not two in a row
  st.template fetch_range<0, LOADS>(0, K);
  u32x4_t second[LOADS];
  static_for<0, LOADS>([&](auto i) { second[decltype(i)::value] = st.template load_one<decltype(i)::value>(min(1, kt_last), K); });
  st.template commit_range<0, LOADS>(lds);
  static_for<0, LOADS>([&](auto i) { st.reg[decltype(i)::value] = second[decltype(i)::value]; });
  __syncthreads();

  Frags4W<T> f0, f1;
  read_range<T, 0, 0, READS>(f0, lds, a_off, b_off, koff);
  for (int kt = 0; kt < kt_all; ++kt) {
    const char* cur = lds + (kt & 1) * T::STAGE_BYTES;
    char* nxt = lds + ((kt + 1) & 1) * T::STAGE_BYTES;
    const int kf = min(kt + 2, kt_last);
    static_for<0, SLOTS>([&](auto sl) {
      constexpr int S = decltype(sl)::value, PART = S / PAIRS, J = S % PAIRS;
      if constexpr (S == 3 * PAIRS) {
        wait_lgkmcnt0();   // own LDS stores of tile kt+1 are done and every read of tile kt has returned
        barrier_no_drain();
      }
      mma_pair<T, J>(acc, (PART & 1) ? f1 : f0);
      // fragment reads: one step ahead, spread over the step's slots; the steps around the barrier
      // read in their first half so that the waits find the data there
      if constexpr (PART == 0) read_range<T, 1, J * READS / PAIRS, (J + 1) * READS / PAIRS>(f1, cur, a_off, b_off, koff);
      if constexpr (PART == 1) read_range<T, 2, J * READS / PAIRS, (J + 1) * READS / PAIRS>(f0, cur, a_off, b_off, koff);
      if constexpr (PART == 2 && J < T::HALF)
        read_range<T, 3, J * READS / T::HALF, (J + 1) * READS / T::HALF>(f1, cur, a_off, b_off, koff);
      if constexpr (PART == 3 && J < T::HALF)
        read_range<T, 0, J * READS / T::HALF, (J + 1) * READS / T::HALF>(f0, nxt, a_off, b_off, koff);
      // register i goes to LDS during the first two steps and is refilled (tile kt+2) later in
      // the iteration: the loads are spread over the whole iteration, since a burst would
      // saturate the address unit and stall the wave
      if constexpr (S < 2 * PAIRS) st.template commit_range<S * LOADS / (2 * PAIRS), (S + 1) * LOADS / (2 * PAIRS)>(nxt);
      if constexpr (S % 2 == 1) st.template fetch_range<(S / 2) * LOADS / (SLOTS / 2), (S / 2 + 1) * LOADS / (SLOTS / 2)>(kf, K);
      __builtin_amdgcn_sched_barrier(0);
    });
  }
  }
}

// Mainloop for tiles whose operands stream from HBM rather than from the L2 (the grouped GEMM's expert
// weights): what bounds such a tile is the bytes a compute unit has in flight, so the two stages above
// (one K tile requested ahead: 32 KiB at the 128 x 128 tile, about 32 GB/s per unit at 2 us of memory
// latency) become a ring of NST stages filled by direct-to-LDS loads, NST - 1 K tiles ahead, one barrier
// per K tile; the matrix work of a K tile (512 cycles at 128 x 128) is short against its loads.
// Requests past the last K tile are out of the buffers' range: zeros are written, memory is not asked.
template <class T, int NST, class ARow, class BRow>
__device__ __forceinline__ void gemm_mainloop_ring(typename T::Acc32& acc, const char* a_base, ARow a_row,
                                                      const char* b_base, BRow b_row, int K, char* lds) {
  static_assert(T::DIRECT && !T::B_KN, "ring staging is written for [N, K] operands loaded straight into LDS");
  constexpr int PAIRS = T::PAIRS, READS = T::READS, LOADS = T::LOADS;
  static_assert((NST - 2) * LOADS <= 63 && NST >= 3, "wait-count immediate");
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 31, lh = lane >> 5;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  const int b_off = T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + lh) ^ swz128(lr)) * 16;
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;
  const int kt_all = (K + 63) / 64;
  Stager4W<T> st;
  st.init(a_base, a_row, b_base, b_row);
#pragma unroll
  for (int j = 0; j < NST - 1; ++j) st.template issue_range<0, LOADS>(j, K, lds + j * T::STAGE_BYTES);
#pragma unroll 1
  for (int kt = 0; kt < kt_all; ++kt) {
    wait_vmcnt<(NST - 2) * LOADS>();   // this wave's part of tile kt has landed (loads return in order)
    barrier_no_drain();                // ... everybody's, and every wave is past its reads of tile kt - 1
    st.template issue_range<0, LOADS>(kt + NST - 1, K, lds + ((kt + NST - 1) % NST) * T::STAGE_BYTES);
    const char* cur = lds + (kt % NST) * T::STAGE_BYTES;
    Frags4W<T> f0, f1;
    read_range<T, 0, 0, READS>(f0, cur, a_off, b_off, koff);
    read_range<T, 1, 0, READS>(f1, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f0); });
    read_range<T, 2, 0, READS>(f0, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f1); });
    read_range<T, 3, 0, READS>(f1, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f0); });
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f1); });
  }
  wait_vmcnt0();   // the requests past the end have completed before the stages are used for anything else
}

// The same ring with the two jobs given to different waves: a work-group of eight waves, waves 0-3 (one per
// SIMD) only read fragments and issue MFMAs, waves 4-7 only issue the loads.  A wave issues in order, so in
// the form above the eight load instructions of a K tile (512 cycles of address-unit time per compute unit)
// and its 512 cycles of matrix work follow one another; here they overlap.  Returns true in the computing
// waves (which hold the accumulators) and false in the loading waves, whose requests have all completed.
template <class T, int NST, class ARow, class BRow>
__device__ __forceinline__ bool gemm_mainloop_ring_split(typename T::Acc32& acc, const char* a_base, ARow a_row,
                                                            const char* b_base, BRow b_row, int K, char* lds) {
  static_assert(T::DIRECT && !T::B_KN, "ring staging is written for [N, K] operands loaded straight into LDS");
  constexpr int PAIRS = T::PAIRS, READS = T::READS, LOADS = T::LOADS;
  static_assert((NST - 2) * LOADS <= 63 && NST >= 3, "wait-count immediate");
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int kt_all = (K + 63) / 64;
  if (wave >= T::NWAVES) {
    Stager4W<T> st;
    st.init(a_base, a_row, b_base, b_row, (int)threadIdx.x - T::THREADS);
#pragma unroll
    for (int j = 0; j < NST - 1; ++j) st.template issue_range<0, LOADS>(j, K, lds + j * T::STAGE_BYTES);
#pragma unroll 1
    for (int kt = 0; kt < kt_all; ++kt) {
      wait_vmcnt<(NST - 2) * LOADS>();   // this wave's part of tile kt has landed (loads return in order)
      barrier_no_drain();                // ... everybody's, and the computing waves are past tile kt - 1
      st.template issue_range<0, LOADS>(kt + NST - 1, K, lds + ((kt + NST - 1) % NST) * T::STAGE_BYTES);
    }
    wait_vmcnt0();
    return false;
  }
  const int wm = wave / 2, wn = wave % 2;
  const int lr = lane & 31, lh = lane >> 5;
  const int a_off = (wm * T::WTM + lr) * T::ROW_BYTES;
  const int b_off = T::A_BYTES + (wn * T::WTN + lr) * T::ROW_BYTES;
  int koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) koff[ks] = ((ks * 2 + lh) ^ swz128(lr)) * 16;
#pragma unroll
  for (int ni = 0; ni < T::NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < T::MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.f;
#pragma unroll 1
  for (int kt = 0; kt < kt_all; ++kt) {
    barrier_no_drain();
    const char* cur = lds + (kt % NST) * T::STAGE_BYTES;
    Frags4W<T> f0, f1;
    read_range<T, 0, 0, READS>(f0, cur, a_off, b_off, koff);
    read_range<T, 1, 0, READS>(f1, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f0); });
    read_range<T, 2, 0, READS>(f0, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f1); });
    read_range<T, 3, 0, READS>(f1, cur, a_off, b_off, koff);
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f0); });
    static_for<0, PAIRS>([&](auto j) { mma_pair<T, decltype(j)::value>(acc, f1); });
    wait_lgkmcnt0();   // every read of tile kt has returned before the next barrier frees its stage
  }
  return true;
}

// Epilogue: each wave turns its accumulators into bf16, parks them in its
// own piece of the (now idle) operand stages, and reads them back row by row so that every
// global store covers whole 128-byte lines (one row = WTN bf16 = SL slots of 16 bytes, read by
// SL lanes; written straight from the MFMA layout, a store instruction would scatter 8-byte
// pieces over 32 rows).  A parked row has SLP >= SL slots (a power of two); the 16-byte slot g
// of row m lives at slot g ^ key(m), which keeps the 8-byte writes (2-way at worst) and the
// 16-byte reads away from bank conflicts.  STREAM: global stores with the streaming hint (for a tile
// that is followed by a release and read much later: nothing dirty is left for the release to write back).
template <class T>
struct ParkedTile {
  static constexpr int SL = T::WTN / 8;            // 16-byte slots of data per row: 16, 12 or 8
  static constexpr int SLP = SL <= 8 ? 8 : 16;     // slots per parked row
  static constexpr int ROW = SLP * 16;             // bytes per parked row
  static_assert(4 * T::WTM * ROW <= T::LDS_BYTES, "the parked tile fits in the operand stages");
  // 128-byte rows pair up in a 256-byte bank window
  __device__ static __forceinline__ int key(int m) { return SLP == 16 ? (m & 15) : ((m >> 1) & 7); }
};

// First half of the epilogue: accumulators -> bf16 -> the wave's piece of the operand stages.
template <class T>
__device__ __forceinline__ void park_tile_bf16(const typename T::Acc& acc, char* lds) {
  typedef ParkedTile<T> P;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  __syncthreads();   // every wave is done reading the operand stages
  char* park = lds + wave * (T::WTM * P::ROW);
  if constexpr (T::X16) {
    // a lane holds, per block, row (lane % 16) and the four columns 4 (lane / 16) .. + 3: half a 16-byte slot
    const int lr = lane & 15, lq = lane >> 4;
#pragma unroll
    for (int mb = 0; mb < T::MB; ++mb) {
      const int m = mb * 16 + lr;
#pragma unroll
      for (int nb = 0; nb < T::NB; ++nb) {
        const int g = nb * 2 + (lq >> 1);
        bf16x4_t v = {(__bf16)acc[nb][mb][0], (__bf16)acc[nb][mb][1], (__bf16)acc[nb][mb][2], (__bf16)acc[nb][mb][3]};
        *(bf16x4_t*)(park + m * P::ROW + ((g ^ P::key(m)) * 16) + (lq & 1) * 8) = v;
      }
    }
    wait_lgkmcnt0();
    return;
  } else {
  const int lr = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < T::MI; ++mi) {
    const int m = mi * 32 + lr;
#pragma unroll
    for (int ni = 0; ni < T::NI; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int g = ni * 4 + q;
        bf16x4_t v = {(__bf16)acc[ni][mi][q * 4 + 0], (__bf16)acc[ni][mi][q * 4 + 1],
                      (__bf16)acc[ni][mi][q * 4 + 2], (__bf16)acc[ni][mi][q * 4 + 3]};
        *(bf16x4_t*)(park + m * P::ROW + ((g ^ P::key(m)) * 16) + lh * 8) = v;
      }
    }
  }
  // the reads that follow are the same wave's: LDS operations of one wave complete in order
  wait_lgkmcnt0();
  }
}

// Second half: the rows m_lo <= m < m_hi of the parked tile (global row numbers; the tile starts at row
// m0, column n0) go to c[m, n] with leading dimension ldc.  May be called several times with different
// windows and destinations.
template <class T, bool STREAM = false>
__device__ __forceinline__ void store_parked_bf16(__bf16* c, size_t ldc, int m0, int n0, int m_lo, int m_hi, int N,
                                                      const char* lds) {
  typedef ParkedTile<T> P;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int wm = wave / 2, wn = wave % 2;
  const char* park = lds + wave * (T::WTM * P::ROW);
  constexpr int ROWS_PER_READ = 64 / P::SLP;
  const int g = lane % P::SLP;
  const int gn = n0 + wn * T::WTN + g * 8;
#pragma unroll 8
  for (int it = 0; it < T::WTM / ROWS_PER_READ; ++it) {
    const int row = it * ROWS_PER_READ + lane / P::SLP;
    const u32x4_t v = *(const u32x4_t*)(park + row * P::ROW + ((g ^ P::key(row)) * 16));
    const int gm = m0 + wm * T::WTM + row;
    if (g < P::SL && gm >= m_lo && gm < m_hi && gn < N) {
      if (STREAM) __builtin_nontemporal_store(v, (u32x4_t*)(c + (size_t)gm * ldc + gn)); else *(u32x4_t*)(c + (size_t)gm * ldc + gn) = v;
    }
  }
}

template <class T, bool STREAM = false>
__device__ __forceinline__ void store_tile_bf16(const typename T::Acc& acc, __bf16* c, size_t ldc, int m0,
                                                    int n0, int M, int N, char* lds) {
  park_tile_bf16<T>(acc, lds);
  store_parked_bf16<T, STREAM>(c, ldc, m0, n0, m0, M, N, lds);
}

}  // namespace ditron
