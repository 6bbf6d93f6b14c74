// Device-side helpers shared by the kernels: signal flags, chunk copies, small utilities.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/ditron.h"

namespace ditron {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

#define DITRON_LDS(p) ((__attribute__((address_space(3))) void*)(p))

__host__ __device__ inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------ signal flags
// A flag is raised with a release store at agent scope after the data it guards, and
// observed with an acquire load at agent scope before the data is read (the paper's
// `wait` + `consume_token` pair and its release `st`).  The eight chiplets have separate
// L2 caches, so nothing weaker than agent scope orders a producer on one chiplet with a
// consumer on another.
__device__ inline void flag_raise(int32_t* flag, int32_t value) {
  __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// One lane polls `count` consecutive flags until each equals `value`; gives up after
// `spin_limit` polls per flag and records the time-out.  Returns with acquire ordering.
__device__ inline void flag_wait_lane(const int32_t* flags, int first, int count, int32_t value,
                                      unsigned spin_limit, int32_t* status) {
  for (int i = 0; i < count; ++i) {
    const int32_t* f = flags + first + i;
    unsigned polls = 0;
    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != value) {
      if (++polls >= spin_limit) {
        status[1] = first + i;
        status[0] = DITRON_ERR_TIMEOUT;
        break;
      }
      __builtin_amdgcn_s_sleep(8);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// One wave waits for `count` flags, one lane per flag: a wait for several flags costs one round
// trip to memory, not one per flag.  Called by all lanes of the wave.
__device__ inline void flag_wait_wave(const int32_t* flags, int first, int count, int32_t value,
                                      unsigned spin_limit, int32_t* status) {
  for (int i = threadIdx.x & 63; i < count; i += 64) {
    const int32_t* f = flags + first + i;
    unsigned polls = 0;
    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != value) {
      if (++polls >= spin_limit) {
        status[1] = first + i;
        status[0] = DITRON_ERR_TIMEOUT;
        break;
      }
      __builtin_amdgcn_s_sleep(8);
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// Whole work-group waits: the first wave polls, the barrier hands the acquired view to the rest.
__device__ inline void flag_wait_block(const int32_t* flags, int first, int count, int32_t value,
                                       unsigned spin_limit, int32_t* status) {
  if (threadIdx.x < 64) flag_wait_wave(flags, first, count, value, spin_limit, status);
  __syncthreads();
}

// ------------------------------------------------------------------ chunk copy
// Copy `bytes` (multiple of 16) from src to dst with 128-bit accesses, the calling
// work-group being part `part` of `nparts` cooperating work-groups.
// U = independent 16-byte loads in flight per lane; all loads of a round are issued before the first store.
// Two forms, each measured against the other where it is used:
//  * STREAM (nothing on the chip reads the copy soon; the MoE gather, consumed by a later launch): a
//    work-group takes contiguous blocks of U * blockDim vectors, dealt to the work-groups in turn, reads them
//    with ordinary loads and stores past the chiplet's L2, so that the flag's release has no dirty lines to
//    write back.  134 MB gather: 5.0 TB/s read + write, what a plain device-to-device copy reaches on the
//    chip; with the streaming hint on the loads, or with the other form, 3.5.
//  * otherwise (GEMM tiles of the same launch are waiting for the data: AllGather-GEMM, GEMM-ReduceScatter):
//    vectors interleaved over the work-groups, loads with the streaming hint (the source is read once and
//    should not displace the operand panels in the L2), ordinary stores.  cfg 2 fused launch: 417 us against
//    455 us with the first form.
template <int U, bool STREAM = false>
__device__ inline void copy_slice_u(void* __restrict__ dst, const void* __restrict__ src, size_t bytes,
                                    int part, int nparts) {
  const size_t n16 = bytes >> 4;
  const u32x4_t* s = (const u32x4_t*)src;
  u32x4_t* d = (u32x4_t*)dst;
  if constexpr (STREAM) {
    const size_t block = (size_t)U * blockDim.x;
    for (size_t b0 = (size_t)part * block; b0 < n16; b0 += (size_t)nparts * block) {
      u32x4_t v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t i = b0 + u * blockDim.x + threadIdx.x;
        if (i < n16) v[u] = s[i];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const size_t i = b0 + u * blockDim.x + threadIdx.x;
        if (i < n16) __builtin_nontemporal_store(v[u], d + i);
      }
    }
  } else {
    const size_t stride = (size_t)nparts * blockDim.x;
    for (size_t i = (size_t)part * blockDim.x + threadIdx.x; i < n16; i += U * stride) {
      u32x4_t v[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (i + u * stride < n16) v[u] = __builtin_nontemporal_load(s + i + u * stride);
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (i + u * stride < n16) d[i + u * stride] = v[u];
    }
  }
}

// A work-group of THREADS threads keeps about 128 KiB of loads in flight whatever its size.
template <int THREADS, bool STREAM = false>
__device__ inline void copy_slice(void* __restrict__ dst, const void* __restrict__ src, size_t bytes,
                                  int part, int nparts) {
  copy_slice_u<(THREADS <= 256 ? 32 : 16), STREAM>(dst, src, bytes, part, nparts);
}

// After every cooperating work-group has finished its slice of a chunk, the last one to
// arrive raises the chunk's flag and leaves the arrival counter at zero for the next call.
// Arrivals are release-only; just the last arrival pays for an acquire (on this chip an
// agent-scope acquire invalidates the chiplet's L2, which the GEMM tiles next door live on).
__device__ inline void publish_after_all(int32_t* counter, int nparts, int32_t* flag, int32_t value) {
  __syncthreads();
  if (nparts == 1) {   // nobody to wait for: the flag's release covers the work-group's stores
    if (threadIdx.x == 0) flag_raise(flag, value);
    return;
  }
  if (threadIdx.x == 0) {
    int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    if (old == nparts - 1) {
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      flag_raise(flag, value);
    }
  }
}

// The emulated peers.  `nchunks` chunks of `chunk_bytes` are delivered by the `nparts` producer
// work-groups (this one is `part`); dst(i) / src(i) / flag(i) / counter(i) give the addresses of
// the chunk at delivery position i.  The producers split into `teams` teams; team t delivers
// chunks t, t + teams, ... one after the other, all its members sharing each copy, and the
// member that finishes a chunk last raises its flag.  One team means strictly sequential
// arrival in delivery order (a ring); as many teams as chunks means everything is in flight
// at once (a full mesh where every peer pushes at the same time).
template <int THREADS, bool STREAM = false, class Dst, class Src, class Flag, class Counter>
__device__ inline void produce_chunks(int nchunks, size_t chunk_bytes, int part, int nparts, int teams,
                                      int32_t epoch, Dst dst, Src src, Flag flag, Counter counter) {
  teams = max(1, min(teams, min(nparts, nchunks)));
  const int team_size = nparts / teams;
  const int team = part / team_size, member = part % team_size;
  if (team >= teams) return;   // left-over work-groups when nparts is not a multiple of teams
  for (int i = team; i < nchunks; i += teams) {
    copy_slice<THREADS, STREAM>(dst(i), src(i), chunk_bytes, member, team_size);
    publish_after_all(counter(i), team_size, flag(i), epoch);
  }
}

// ------------------------------------------------------------------ tile ordering
// Linear tile id -> (pid_m, pid_n), tile rows in groups of group_m with the row index
// running fastest inside a group (paper, first lines of the AllGather-GEMM consumer).
__host__ __device__ inline int imin(int a, int b) { return a < b ? a : b; }

__host__ __device__ inline void grouped_order(int pid, int npm, int npn, int group_m, int& pid_m, int& pid_n) {
  const int in_group = group_m * npn;
  const int first_m = (pid / in_group) * group_m;
  const int size_m = imin(npm - first_m, group_m);
  const int r = pid % in_group;
  pid_m = first_m + r % size_m;
  pid_n = r / size_m;
}

// ------------------------------------------------------------------ tile rows across nodes
// Position in the visiting order -> tile row, for `nnodes` nodes of world/nnodes ranks each
// (paper, Appendix "Swizzle", first listing for the gather order and second for the scatter
// order).  Nodes are visited starting with the own node (gather) or the next one (scatter);
// inside a node the rows are rotated to start at the own local rank's rows (gather) or the
// next local rank's (scatter).  A tile row that straddles two nodes belongs to exactly one
// of them; which one depends on the visit position and differs between the two orders.
// With one node both reduce to the plain rotations used by the kernels.
enum { kOrderGather = 0, kOrderScatter = 1 };

// Tile rows [t_lo, t_lo + size) owned by the node visited at position `pos`.  A tile row that holds
// rows of two neighbouring nodes is owned by the one visited later in gather order (the data of
// both must have arrived) and by the one visited earlier in scatter order (it is computed as early
// as possible for both).  The node below in id is visited right before this one, except at the
// first position; the node above right after it, except at the last.
__host__ __device__ inline void node_tile_rows(int pos, int m, int nnodes, int block_m, int node_start, int mode,
                                               int& t_lo, int& size) {
  const int m_node = m / nnodes;
  const int node = (pos + node_start) % nnodes;
  const int lo = m_node * node, hi = m_node * (node + 1);
  t_lo = lo / block_m;
  int t_hi = (hi - 1) / block_m;
  const bool shares_first = lo != 0 && (lo - 1) / block_m == t_lo;
  const bool shares_last = hi != m && hi / block_m == t_hi;
  const bool after_lower = pos != 0, after_upper = pos == nnodes - 1;
  const bool later_owns = mode == kOrderGather;
  if (shares_first && after_lower != later_owns) ++t_lo;
  if (shares_last && after_upper != later_owns) --t_hi;
  size = t_hi - t_lo + 1;
}

__host__ __device__ inline int tile_row_across_nodes(int position, int m, int rank, int world, int nnodes, int block_m,
                                                     int mode) {
  const int local_world = world / nnodes;
  const int node_id = rank / local_world, local_rank = rank % local_world;
  const int m_r = m / world, m_node = m / nnodes;
  const int node_start = (node_id + (mode == kOrderScatter ? 1 : 0)) % nnodes;
  // the visit position the tile falls in
  int before = 0, pos = -1, size = 0;
  for (int p = 0; p < nnodes; ++p) {
    int lo, sz;
    node_tile_rows(p, m, nnodes, block_m, node_start, mode, lo, sz);
    if (position < before + sz) { pos = p; size = sz; break; }
    before += sz;
  }
  if (pos < 0) return position;   // past the swizzled range: cannot happen while the blocks cover every tile row
  const int nid = (pos + node_start) % nnodes;
  // first tile row of that node = sizes of the nodes with a smaller id
  int node_offset = 0;
  for (int p = 0; p < nnodes; ++p) {
    if ((p + node_start) % nnodes < nid) {
      int lo, sz;
      node_tile_rows(p, m, nnodes, block_m, node_start, mode, lo, sz);
      node_offset += sz;
    }
  }
  const int first_row = mode == kOrderGather ? cdiv(m_node * nid + m_r * local_rank, block_m)
                                             : (m_node * nid + m_r * (local_rank + 1)) / block_m;
  const int rank_offset = first_row > node_offset ? first_row - node_offset : 0;
  return node_offset + (position - before + rank_offset) % size;
}

// Work-group index -> linear tile id.  The dispatcher deals work-groups round-robin to the
// chiplets; inside every block of num_xcd*per_xcd tiles, chiplet x receives a run of
// consecutive tile ids, so tiles that share operand panels share an L2, while blocks stay in
// schedule order.
__host__ __device__ inline int xcd_remap(int wg, int ntiles, int num_xcd, int per_xcd) {
  if (num_xcd <= 1) return wg;
  const int block = num_xcd * per_xcd;
  const int base = (wg / block) * block;
  const int size = imin(block, ntiles - base);
  const int local = wg - base;
  const int x = local % num_xcd, j = local / num_xcd;
  const int q = size / num_xcd, rem = size % num_xcd;
  // chiplets 0..rem-1 own q+1 work-groups of this block, the rest own q
  const int start = x * q + imin(x, rem);
  return base + start + j;
}

// ------------------------------------------------------------------ work-group -> tile
// The whole index arithmetic of a GEMM work-group, shared by the kernels and by the host evaluation
// of the schedule: chiplet remap, grouped order, then the rank rotation (across nodes: the multi-node
// order) and the span of shards (gather) or segments (scatter) the tile's rows touch.
struct TileOrder {
  int npm, npn, group_m, num_xcd, per_xcd;
};
struct TileSpan {
  int pid_m, pid_n, first, last;
};
__host__ __device__ inline TileSpan tile_of_workgroup(int wg, const TileOrder& o, int mode, int m, int m_per_rank,
                                                      int rank, int world, int nnodes, int block_m) {
  const int pid = xcd_remap(wg, o.npm * o.npn, o.num_xcd, o.per_xcd);
  TileSpan t;
  grouped_order(pid, o.npm, o.npn, o.group_m, t.pid_m, t.pid_n);
  if (nnodes > 1) {
    t.pid_m = tile_row_across_nodes(t.pid_m, m, rank, world, nnodes, block_m, mode);
  } else if (mode == kOrderGather) {
    // start on the rows of the rank's own shard, then follow the ring
    t.pid_m = (t.pid_m + cdiv(m_per_rank * rank, block_m)) % o.npm;
  } else {
    // the next rank's segment first, the own segment last
    t.pid_m = (t.pid_m + ((rank + 1) * m_per_rank) / block_m) % o.npm;
  }
  const int m0 = t.pid_m * block_m;
  t.first = m0 / m_per_rank;
  t.last = (imin(m0 + block_m, m) - 1) / m_per_rank;
  return t;
}

}  // namespace ditron
