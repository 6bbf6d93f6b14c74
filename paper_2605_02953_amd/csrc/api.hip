// Entry points that are not tied to one operator: sizes, tile choice, spin limit, status
// strings, and the external chunk publisher used by tests and by integrations that bring
// their own transport.
#include "launch.h"

namespace ditron {

struct PublishParams {
  void* dst[64];
  const void* src[64];
  size_t bytes[64];
  int flag_index[64];
  int32_t* signals;
  int n;
  int32_t epoch;
  unsigned delay_cycles;
};

// A single work-group walks the chunks in order: optional idle time, copy, then the flag.
__global__ __launch_bounds__(1024) void publish_chunks_kernel(const PublishParams p) {
  for (int i = 0; i < p.n; ++i) {
    if (p.delay_cycles) {
      const unsigned long long t0 = wall_clock64();
      while (wall_clock64() - t0 < p.delay_cycles) __builtin_amdgcn_s_sleep(32);
    }
    copy_slice<1024>(p.dst[i], p.src[i], p.bytes[i], 0, 1);
    __syncthreads();
    if (threadIdx.x == 0) flag_raise(p.signals + p.flag_index[i], p.epoch);
  }
}
}  // namespace ditron

using namespace ditron;

extern "C" size_t ditron_signal_words(int world, int chunks) {
  if (world < 1 || chunks < 1) return 0;
  // flags [world] + per-rank counters [world] + chunk flags [world*chunks] + chunk counters [world*chunks]
  // + the flags of the MoE routing work-groups (which sit behind a one-chunk layout)
  return (size_t)world * 2 + (size_t)world * chunks * 2 + 16;
}

extern "C" ditron_status_t ditron_tile_config(int op, int m, int n, int k, int dtype, const ditron_tuning_t* tuning,
                                              int out[DITRON_TILE_CONFIG_WORDS]) {
  if (!out || m <= 0 || n <= 0 || k <= 0 || op < 0 || op > 4) return DITRON_ERR_INVALID_ARG;
  if (dtype != DITRON_BF16 && dtype != DITRON_FP8_E4M3) return DITRON_ERR_INVALID_ARG;
  if (dtype == DITRON_FP8_E4M3 && op != 0) return DITRON_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning, 1);
  if (!tune.valid) return DITRON_ERR_INVALID_ARG;
  const bool decode = dtype == DITRON_FP8_E4M3 || (op == 0 && bf16_ag_is_decode_shaped(m, n));
  TileChoice t = decode ? choose_tile_decode(m, n, k) : choose_tile(m, n, k, op == 0);
  int splits = 1;
  if (decode) {
    const DecodePlan plan = plan_decode(m, n, k * (dtype == DITRON_BF16 ? 2 : 1), tune.decode_variant);
    t.block_m = plan.block_m;
    t.block_n = plan.block_n;
    splits = plan.splits;
    if (plan.variant != 1) t.num_xcd = t.per_xcd = 0;   // the split-K kernel applies no remap to the tile ids
  }
  if (op == 2) {  // the grouped GEMM has its own row tile; its column block is chosen per call; m is max_rows
    t.big = false;
    t.block_m = kMoeBlockM;
    t.block_n = 0;
    t.threads = 256;
  }
  out[0] = t.block_m;
  out[1] = t.block_n;
  out[2] = t.group_m;
  out[3] = t.num_xcd;
  out[4] = t.per_xcd;
  out[5] = t.block_n ? cdiv(m, t.block_m) * cdiv(n, t.block_n) : 0;
  out[6] = t.threads;
  // operand staging of the tile engine: 1 = straight into LDS (256 x 256 tiles, B stored [n, k])
  out[7] = (!decode && op != 2 && op != 4 && t.big) ? 1 : 0;
  out[8] = splits;
  out[9] = 0;
  return DITRON_OK;
}

extern "C" size_t ditron_ag_gemm_workspace_bytes(int m_per_rank, int n, int k, int world, int dtype, int b_layout,
                                                 const ditron_tuning_t* tuning) {
  if (m_per_rank <= 0 || n <= 0 || k <= 0 || world < 1 || world > DITRON_MAX_WORLD) return 0;
  if (dtype != DITRON_BF16 && dtype != DITRON_FP8_E4M3) return 0;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return 0;
  const Tuning tune = resolve_tuning(tuning, world);
  if (!tune.valid) return 0;
  const int esize = dtype == DITRON_BF16 ? 2 : 1;
  const int m = world * m_per_rank;
  const size_t gathered = (size_t)m * k * esize;
  const bool decode = dtype == DITRON_FP8_E4M3 || (b_layout == DITRON_B_NK && bf16_ag_is_decode_shaped(m, n));
  if (!decode) return gathered;
  // decode-shaped problems: the partial tiles of the split contraction follow the gathered operand
  const DecodePlan plan = plan_decode(m, n, k * esize, tune.decode_variant);
  return plan.partial_bytes ? align256(gathered) + plan.partial_bytes : gathered;
}

extern "C" size_t ditron_moe_workspace_bytes(int tokens_per_rank, int hidden, int world) {
  if (tokens_per_rank <= 0 || hidden <= 0 || world < 1 || world > DITRON_MAX_WORLD) return 0;
  return align256((size_t)world * tokens_per_rank * hidden * 2) + DITRON_MOE_ROUTE_SCRATCH_BYTES;
}

extern "C" ditron_status_t ditron_schedule_dump(int op, int m, int n, int k, int world, int rank, int dtype, int b_layout,
                                                const ditron_tuning_t* tuning, int32_t* out, int capacity, int* count) {
  if ((op != 0 && op != 1 && op != 3) || m <= 0 || n <= 0 || k <= 0 || !count || capacity < 0 || (capacity && !out))
    return DITRON_ERR_INVALID_ARG;
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (op != 3 && m % world != 0) return DITRON_ERR_INVALID_ARG;
  if (dtype != DITRON_BF16 && dtype != DITRON_FP8_E4M3) return DITRON_ERR_INVALID_ARG;
  if (b_layout != DITRON_B_KN && b_layout != DITRON_B_NK) return DITRON_ERR_INVALID_ARG;
  if (dtype == DITRON_FP8_E4M3 && (op != 0 || b_layout != DITRON_B_NK)) return DITRON_ERR_UNSUPPORTED;
  const Tuning tune = resolve_tuning(tuning, op == 3 ? 1 : world);
  if (!tune.valid) return DITRON_ERR_INVALID_ARG;
  const bool decode = op == 0 && (dtype == DITRON_FP8_E4M3 || (b_layout == DITRON_B_NK && bf16_ag_is_decode_shaped(m, n)));
  TileChoice tc = decode ? choose_tile_decode(m, n, k) : choose_tile(m, n, k, op == 0 && b_layout == DITRON_B_NK);
  int splits = 1;
  if (decode) {
    const DecodePlan plan = plan_decode(m, n, k * (dtype == DITRON_BF16 ? 2 : 1), tune.decode_variant);
    tc.block_m = plan.block_m;
    tc.block_n = plan.block_n;
    splits = plan.splits;
    if (plan.variant != 1) tc.num_xcd = tc.per_xcd = 0;
  }
  const TileOrder o{cdiv(m, tc.block_m), cdiv(n, tc.block_n), tc.group_m, tc.num_xcd, tc.per_xcd};
  const int ntiles = o.npm * o.npn;
  *count = ntiles * splits;
  if (*count > capacity) return DITRON_ERR_WORKSPACE;
  if (op != 3 && tune.num_nodes > 1 &&
      !node_order_is_bijection(m, tc.block_m, world, tune.num_nodes, rank, op == 0 ? kOrderGather : kOrderScatter))
    return DITRON_ERR_UNSUPPORTED;
  for (int wg = 0; wg < ntiles; ++wg) {
    int32_t* rec = out + (size_t)DITRON_SCHEDULE_WORDS * wg * splits;
    if (op == 3) {
      int pid_m, pid_n;
      grouped_order(xcd_remap(wg, ntiles, o.num_xcd, o.per_xcd), o.npm, o.npn, o.group_m, pid_m, pid_n);
      rec[0] = pid_m; rec[1] = pid_n; rec[2] = 0; rec[3] = 0;
    } else {
      const TileSpan t = tile_of_workgroup(wg, o, op == 0 ? kOrderGather : kOrderScatter, m, m / world, rank, world,
                                           tune.num_nodes, tc.block_m);
      // the splits of a tile share its record
      for (int ks = 0; ks < splits; ++ks) {
        int32_t* r = rec + DITRON_SCHEDULE_WORDS * ks;
        r[0] = t.pid_m; r[1] = t.pid_n; r[2] = t.first; r[3] = t.last;
      }
    }
  }
  return DITRON_OK;
}

extern "C" ditron_status_t ditron_moe_tile_choice(int total_tokens, int top_k, int num_experts, int num_local_experts,
                                                  int inter, int out[2]) {
  if (!out || total_tokens <= 0 || top_k <= 0 || num_experts <= 0 || num_local_experts <= 0 ||
      num_local_experts > num_experts || inter <= 0)
    return DITRON_ERR_INVALID_ARG;
  const MoeTile t = choose_moe_tile(moe_expected_rows(total_tokens, top_k, num_experts, num_local_experts), num_local_experts, inter);
  out[0] = t.block_m;
  out[1] = t.block_n;
  return DITRON_OK;
}

extern "C" ditron_status_t ditron_tile_row_order(int op, int m, int block_m, int world, int nnodes, int rank, int* out) {
  if (!out || (op != 0 && op != 1) || m <= 0 || block_m <= 0) return DITRON_ERR_INVALID_ARG;
  if (world < 1 || world > DITRON_MAX_WORLD || rank < 0 || rank >= world) return DITRON_ERR_INVALID_ARG;
  if (nnodes < 1 || world % nnodes != 0 || m % world != 0) return DITRON_ERR_INVALID_ARG;
  const int npm = cdiv(m, block_m);
  for (int t = 0; t < npm; ++t)
    out[t] = tile_row_across_nodes(t, m, rank, world, nnodes, block_m, op == 0 ? kOrderGather : kOrderScatter);
  return DITRON_OK;
}

extern "C" const char* ditron_status_string(int status) {
  switch (status) {
    case DITRON_OK: return "ok";
    case DITRON_ERR_INVALID_ARG: return "invalid argument";
    case DITRON_ERR_UNSUPPORTED: return "unsupported shape, layout or dtype";
    case DITRON_ERR_WORKSPACE: return "workspace too small";
    case DITRON_ERR_HIP: return "HIP launch failed";
    case DITRON_ERR_TIMEOUT: return "signal wait timed out";
    default: return "unknown status";
  }
}

extern "C" ditron_status_t ditron_publish_chunks(void* const* dst, const void* const* src, const size_t* bytes,
                                                 const int* flag_index, int32_t* signals, int n, int32_t epoch,
                                                 unsigned delay_cycles, void* stream) {
  if (n < 0 || n > 64 || !signals) return DITRON_ERR_INVALID_ARG;
  if (n == 0) return DITRON_OK;
  if (!dst || !src || !bytes || !flag_index) return DITRON_ERR_INVALID_ARG;
  PublishParams p{};
  for (int i = 0; i < n; ++i) {
    if ((bytes[i] & 15u) || flag_index[i] < 0) return DITRON_ERR_INVALID_ARG;
    if (bytes[i] && (!dst[i] || !src[i] || !aligned16(dst[i]) || !aligned16(src[i]))) return DITRON_ERR_INVALID_ARG;
    p.dst[i] = dst[i];
    p.src[i] = src[i];
    p.bytes[i] = bytes[i];
    p.flag_index[i] = flag_index[i];
  }
  p.signals = signals;
  p.n = n;
  p.epoch = epoch;
  p.delay_cycles = delay_cycles;
  hipLaunchKernelGGL(publish_chunks_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, p);
  return hipGetLastError() == hipSuccess ? DITRON_OK : DITRON_ERR_HIP;
}
