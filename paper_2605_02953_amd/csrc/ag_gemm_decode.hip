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
  int num_producers, teams;
  unsigned spin_limit;
  int wait;   // 0: every shard is resident, the flags are not looked at
  int group_m, num_xcd, per_xcd, npm, npn;
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
  if (p.schedule && threadIdx.x == 0) {
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

  // tile indices past the end re-load the last tile into a free stage: the number of loads per
  // iteration stays fixed, which is what the in-order wait counts below rely on
  auto issue_a = [&](int kt) {
    const int kte = min(kt, kt_all - 1);
    char* stage = lds_a + (kt % T::NA) * T::A_STAGE;
#pragma unroll
    for (int i = 0; i < T::A_LOADS; ++i) {
      const char* src = a_ptr[i] + (size_t)kte * T::BK;
      if (kte * T::BK + a_kc[i] >= K) src = (const char*)&kZeroChunk;
      __builtin_amdgcn_global_load_lds(src, DITRON_LDS(stage + (wave * T::A_LOADS + i) * 1024), 16, 0, 0);
    }
  };
  auto issue_b = [&](int kt) {
    const int kte = min(kt, kt_all - 1);
    char* stage = lds_b + (kt % T::NB) * T::B_STAGE;
    const char* src = b_ptr + (size_t)kte * T::BK;
    if (kte * T::BK + b_kc >= K) src = (const char*)&kZeroChunk;
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

}  // namespace ditron

using namespace ditron;

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
  p.schedule = (flags & DITRON_DUMP_SCHEDULE) ? schedule_out : nullptr;
  p.m_per_rank = m_per_rank;
  p.m = m_per_rank * world;
  p.n = n;
  p.k = k;
  p.world = world;
  p.rank = rank;
  p.nnodes = tune.num_nodes;
  p.epoch = epoch;
  p.spin_limit = tune.spin_limit;
  p.wait = producer_mode(flags) != Mode::kPreset;
  TileChoice tc = choose_tile_decode(p.m, n, k);
  if (p.nnodes > 1 && !node_order_is_bijection(p.m, tc.block_m, world, p.nnodes, rank, kOrderGather))
    return DITRON_ERR_UNSUPPORTED;
  p.group_m = tc.group_m;
  p.num_xcd = tc.num_xcd;
  p.per_xcd = tc.per_xcd;
  const ProducerPlan pl = plan_producers((size_t)p.m * k * (bf16 ? 2 : 1), world);
  p.num_producers = emulate ? pl.producers : 0;
  p.teams = pl.teams;
  p.npm = cdiv(p.m, DecodeTile::BM);
  p.npn = cdiv(p.n, DecodeTile::BN);
  auto kern = bf16 ? ag_gemm_decode_kernel<true> : ag_gemm_decode_kernel<false>;
  if (!(bf16 ? set_dynamic_lds<ag_gemm_decode_kernel<true>>(DecodeTile::LDS_BYTES)
             : set_dynamic_lds<ag_gemm_decode_kernel<false>>(DecodeTile::LDS_BYTES)))
    return DITRON_ERR_HIP;
  const unsigned grid = (unsigned)(p.num_producers + p.npm * p.npn);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(DecodeTile::THREADS), DecodeTile::LDS_BYTES, (hipStream_t)stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}
