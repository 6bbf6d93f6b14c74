// Host-side helpers shared by the entry points: argument checks, tile choice, launch set-up.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <algorithm>
#include <atomic>
#include "../../include/ditron.h"
#include "gemm_core.h"

namespace ditron {

// 256x256 output tile for B stored [N, K]: 128x128 per wave, operands loaded straight into a ring of five LDS
// pieces (160 KiB), 16 x 16 x 32 MFMA.  (Measured with emulated peers against the same tile with register
// staging, two LDS stages and 32 x 32 x 16 MFMA, which it replaced: 5-9 % faster at K 3584 and 8192, 12 % faster at
// 16384, 6 % faster at 3696, whose last K tile is ragged.)
typedef GemmTile4W<256, 256, false, true, true> TileBigDirect;
// The same with 224 and 192 columns: fewer columns per tile for problems whose 256-column tiling leaves the last round
// of 256 units partly empty (choose_tile).
typedef GemmTile4W<256, 224, false, true, true> TileBigDirect224;
typedef GemmTile4W<256, 192, false, true, true> TileBigDirect192;
// 128x128 output tile: 64x64 per wave, 64 KiB of LDS; for problems with too few 256x256 tiles
// to fill the chip.
typedef GemmTile4W<128, 128> TileSmall;
// The same two sizes for B stored [K, N] (register staging, two LDS stages, 32 x 32 x 16 MFMA, as the 128x128 tile).
typedef GemmTile4W<256, 256, true> TileBigKN;
typedef GemmTile4W<128, 128, true> TileSmallKN;
// The MoE grouped GEMM: 4 waves as 2 x 2.  An expert's rows are padded to whole row tiles, so the row
// tile is 128 unless the experts are large or the 128-row tiles would need more rounds (choose_moe_tile).
constexpr int kMoeBlockM = 128;   // the smallest row tile: what the upper bound on the tile count assumes
struct MoeTile {
  int block_m, block_n;
};
// Column block for 128-row tiles.  The number of row tiles is only known on the device, so
// the host works from the expectation under even routing (rows / 128 plus half a tile of
// padding per expert).  If some width gives one tile per compute unit at most, with one row
// tile more than expected still fitting, the narrowest such width: in a single round the time
// is one tile's, and that is bound by the bytes a compute unit can load, (128 + width) * K
// (measured with streamed weights at 20 row tiles x 1536 columns: 62, 72, 74 us for 128, 192,
// 256).  With several rounds the flops decide: the width that pads `inter` least, the wider
// one on a tie (measured: 176 columns 126, 108, 122 us; 256 columns 130, 142, 130 us).
inline int choose_moe_block_n(long expected_rows, int num_local_experts, int inter) {
  const long row_tiles = cdiv((int)std::min<long>(expected_rows, 1 << 30), kMoeBlockM) + (num_local_experts + 1) / 2;
  const int widths[3] = {128, 192, 256};
  for (int w : widths)
    if ((row_tiles + 1) * cdiv(inter, w) <= 256) return w;
  int best = 256;
  for (int w : widths)
    if (cdiv(inter, w) * w < cdiv(inter, best) * best || (cdiv(inter, w) * w == cdiv(inter, best) * best && w > best)) best = w;
  return best;
}
// Row tile.  What a tile costs is the bytes its compute unit loads, (rows + columns) * K, times the rounds
// the launch needs on 256 units; the 256-row tile has two LDS stages instead of a ring fed by loading waves,
// which makes its loads about 1.3 times slower (measured: 64 experts x 768 rows x 256 columns, 416 tiles of
// 128 rows in two rounds against 224 of 256 rows in one: 100 against 85 us for the whole call; 60 experts x
// 546 rows x 176 columns: 97 against 94 us).  From 1024 rows per expert on the 256-row tile is also ahead
// on matrix work (fewer loads per MFMA, little padding).
inline MoeTile choose_moe_tile(long expected_rows, int num_local_experts, int inter) {
  const MoeTile small{kMoeBlockM, choose_moe_block_n(expected_rows, num_local_experts, inter)};
  const MoeTile big{256, inter <= 128 ? 128 : 256};
  if (expected_rows / num_local_experts >= 1024) return big;
  const long rows = std::min<long>(expected_rows, 1 << 30);
  auto per_unit = [&](const MoeTile& t) {
    const long tiles = ((rows + t.block_m - 1) / t.block_m + (num_local_experts + 1) / 2) * cdiv(inter, t.block_n);
    return ((tiles + 255) / 256) * (t.block_m + std::min(t.block_n, inter));
  };
  return 13 * per_unit(big) < 10 * per_unit(small) ? big : small;
}
// rows routed to the local experts if every expert received the same number of assignments
inline long moe_expected_rows(long total_tokens, int top_k, int num_experts, int num_local_experts) {
  return total_tokens * top_k * num_local_experts / num_experts;
}

struct TileChoice {
  bool big;
  int block_m, block_n, threads;
  int group_m;    // GROUP_SIZE_M of the grouped tile order
  int num_xcd;    // chiplets assumed by the work-group remap (0: no remap)
  int per_xcd;    // consecutive tiles handed to one chiplet inside a remap block
};

// What a launch of `tiles` tiles of 256 x block_n costs, in units of a full round of 256 x 256 tiles: the work of a
// tile times the rounds, a last round that fills the fraction x of the chip counting 0.55 + 0.45 x (measured: the
// 192 tiles of cfg 2's second round take 0.886 of the time of the 256 of its first, the chip being power-limited);
// a 224-column tile loads 3 % more bytes per flop, a 192-column tile 7 %.
inline double tiling_cost(long tiles, int block_n) {
  const double work = block_n / 256.0 * (block_n == 256 ? 1.0 : block_n == 224 ? 1.03 : 1.07);
  const long full = tiles / 256, rest = tiles % 256;
  return work * ((double)full + (rest ? 0.55 + 0.45 * (double)rest / 256.0 : 0.0));
}

// narrow_ok: the caller has the 224-column tile (AllGather-GEMM with B stored [N, K]; the column counts of the
// GEMM-ReduceScatter and GEMM + AllReduce shapes of the paper's tables are whole rounds of 256-column tiles)
inline TileChoice choose_tile(int m, int n, int /*k*/, bool narrow_ok = false) {
  TileChoice t{};
  const long tiles_big = (long)cdiv(m, 256) * cdiv(n, 256);
  t.big = tiles_big >= 192;
  t.block_m = t.block_n = t.big ? 256 : 128;
  if (t.big && narrow_ok) {
    double best = 0.98 * tiling_cost(tiles_big, 256);
    for (int bn : {224, 192}) {
      const double c = tiling_cost((long)cdiv(m, 256) * cdiv(n, bn), bn);
      if (c < best) { best = c; t.block_n = bn; }
    }
  }
  t.threads = t.big ? TileBigDirect::THREADS : TileSmall::THREADS;
  t.group_m = 4;
  t.num_xcd = 8;
  t.per_xcd = 32;
  return t;
}

// Decode-shaped AllGather-GEMM (fp8 always; bf16 when the 128 x 128 tiles of the tile engine would not
// cover half the chip and B is stored [n, k]): one tile shape, 128 rows x 32 columns, 4 computing waves +
// 4 loading waves.
inline bool bf16_ag_is_decode_shaped(int m, int n) { return (long)cdiv(m, 128) * cdiv(n, 128) <= 128; }
inline TileChoice choose_tile_decode(int /*m*/, int /*n*/, int /*k*/) {
  TileChoice t{};
  t.big = false;
  t.block_m = 128;
  t.block_n = 32;
  t.threads = 512;
  t.group_m = 4;
  t.num_xcd = 8;
  t.per_xcd = 32;
  return t;
}

// Decode-shaped problems: which kernel, tile and K split.  Variant 1 is the 128 x 32 tile over the whole
// contraction; 2 / 3 are 128 x 128 / 128 x 64 tiles with the contraction split over S work-groups; 4 is the
// per-shard form, 16-row tiles (one shard's rows at the decode shape: a tile waits for that shard only).
// S doubles while the grid stays within one work-group per compute unit, at most 8, and every split keeps at
// least four 128-byte K tiles.
struct DecodePlan {
  int variant, block_m, block_n, splits, kt_per_split, ntiles;
  size_t partial_bytes;   // partial tiles (8 bytes per element: fp32 value + epoch), behind the gathered operand in the workspace
};
inline DecodePlan plan_decode(int m, int n, int k_bytes, int variant) {
  DecodePlan d{};
  d.variant = variant == 0 ? 2 : variant;
  d.block_m = d.variant == 4 ? 16 : 128;
  d.block_n = d.variant == 1 ? 32 : (d.variant == 3 ? 64 : 128);
  d.ntiles = cdiv(m, d.block_m) * cdiv(n, d.block_n);
  const int kt = cdiv(k_bytes, 128);
  d.splits = 1;
  if (d.variant != 1)
    while ((long)d.ntiles * d.splits * 2 <= 256 && d.splits * 2 <= 8 && kt / (d.splits * 2) >= 4) d.splits *= 2;
  d.kt_per_split = cdiv(kt, d.splits);
  d.partial_bytes = d.splits > 1 ? (size_t)d.ntiles * d.splits * d.block_m * d.block_n * 2 * sizeof(float) : 0;
  return d;
}
inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// How many work-groups play the peers, and into how many teams they split (= chunks in flight
// at once).  On one GPU the copies are compute-unit work, so the cheapest emulation delivers
// everything as early and as fast as possible: enough work-groups to saturate HBM for a large
// transfer (about half a MiB each, at most one per compute unit), and as many teams as chunks,
// which is also how a full mesh of links behaves (every peer pushes at the same time).
struct ProducerPlan {
  int producers, teams;
};
inline ProducerPlan plan_producers(size_t total_bytes, int nchunks) {
  ProducerPlan pl{};
  size_t want = (total_bytes + (512u << 10) - 1) / (512u << 10);
  want = (want + 7) / 8 * 8;
  pl.producers = (int)(want < 8 ? 8 : (want > 256 ? 256 : want));
  pl.teams = nchunks < pl.producers ? nchunks : pl.producers;
  if (pl.teams < 1) pl.teams = 1;
  return pl;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The tile loaders address an operand with 32-bit byte offsets, and the buffer-addressed
// loaders reserve offsets from 0x7ffffff0 up as "out of range, reads zero".
inline bool fits_32bit(size_t rows, size_t cols, size_t esize) { return rows * cols * esize < 0x7ffffff0ull; }

// With more than one node the tile-row order comes from the paper's multi-node listings; a shape
// for which they do not visit every tile row exactly once is refused.
inline bool node_order_is_bijection(int m, int block_m, int world, int nnodes, int rank, int mode) {
  const int npm = cdiv(m, block_m);
  constexpr int kMaxRows = 1 << 16;   // one bit per tile row on the stack: the check allocates nothing
  if (npm > kMaxRows) return false;
  uint64_t seen[kMaxRows / 64] = {0};
  for (int t = 0; t < npm; ++t) {
    const int r = tile_row_across_nodes(t, m, rank, world, nnodes, block_m, mode);
    if (r < 0 || r >= npm || (seen[r >> 6] >> (r & 63)) & 1) return false;
    seen[r >> 6] |= 1ull << (r & 63);
  }
  return true;
}

inline bool is_permutation(const int* v, int n) {
  bool seen[DITRON_MAX_WORLD] = {false};
  for (int i = 0; i < n; ++i) {
    if (v[i] < 0 || v[i] >= n || seen[v[i]]) return false;
    seen[v[i]] = true;
  }
  return true;
}

// Kernels with more than 64 KiB of dynamic LDS need the limit raised, once per (kernel, device): the
// outcome is remembered per kernel (one bit per device), so the driver call is not paid on every launch.
template <auto Kernel>
inline bool set_dynamic_lds(int bytes) {
  static std::atomic<uint64_t> configured{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  const uint64_t bit = 1ull << (dev & 63);
  if (configured.load(std::memory_order_acquire) & bit) return true;
  if (hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return false;
  configured.fetch_or(bit, std::memory_order_release);
  return true;
}

// Per-call options with the defaults filled in.
struct Tuning {
  int num_nodes;
  unsigned spin_limit;
  int decode_variant;
  int moe_route_groups;
  bool valid;
};
inline Tuning resolve_tuning(const ditron_tuning_t* t, int world) {
  Tuning r{1, 1u << 20, 0, 0, true};
  if (!t) return r;
  if (t->num_nodes < 0 || t->num_nodes > DITRON_MAX_WORLD || t->decode_variant < 0 || t->decode_variant > 4) r.valid = false;
  if (t->moe_route_groups < 0 || t->moe_route_groups > 8) r.valid = false;
  for (int v : t->reserved) r.valid = r.valid && v == 0;
  if (t->num_nodes > 0) r.num_nodes = t->num_nodes;
  if (t->spin_limit) r.spin_limit = t->spin_limit;
  r.decode_variant = t->decode_variant;
  r.moe_route_groups = t->moe_route_groups;
  if (world % r.num_nodes != 0) r.valid = false;
  return r;
}

// Exactly one of the three producer modes.
enum class Mode { kInvalid, kEmulate, kExternal, kPreset };
inline Mode producer_mode(unsigned flags) {
  switch (flags & (DITRON_EMULATE_PRODUCER | DITRON_EXTERNAL_PRODUCER | DITRON_FLAGS_PRESET)) {
    case DITRON_EMULATE_PRODUCER: return Mode::kEmulate;
    case DITRON_EXTERNAL_PRODUCER: return Mode::kExternal;
    case DITRON_FLAGS_PRESET: return Mode::kPreset;
    default: return Mode::kInvalid;
  }
}

}  // namespace ditron

extern "C" ditron_status_t ditron_ag_gemm_decode(const void* const* a_shards, const void* b, int b_layout, void* c,
                                                 const float* a_scales, const float* b_scales, void* workspace,
                                                 int32_t* signals, int32_t* status, int32_t* schedule_out,
                                                 const int* arrival_order, int m_per_rank, int n, int k, int world,
                                                 int rank, int dtype, int32_t epoch, unsigned flags,
                                                 const ditron_tuning_t* tuning, void* stream);
