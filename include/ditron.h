/*
 * ditron.h -- C ABI of the MI355X (gfx950) fused communication + GEMM kernels.
 *
 * One GPU's share of the tensor-parallel operators below, with the other ranks' shards
 * resident in the same GPU's memory and published, chunk by chunk with one int32 signal
 * flag each, in the order the peer ranks would deliver them:
 *
 *   ditron_ag_gemm              AllGather-GEMM          (paper, Appendix "AllGather GEMM")
 *   ditron_gemm_rs              GEMM-ReduceScatter      (paper, Appendix "GEMM Reduce-Scatter")
 *   ditron_gemm_rs_fuse_scatter the same with the scatter fused into the GEMM's stores
 *   ditron_moe_ag_grouped_gemm  AllGather + grouped GEMM over local experts
 *                               (paper, kernel list "ag_group_gemm"; Appendix "Swizzle", third listing)
 *   ditron_moe_grouped_gemm_rs  MoE down-projection (grouped GEMM + top-k combine) + ReduceScatter
 *   ditron_gemm_ar              GEMM + AllReduce, every tile reduced on every rank
 *   ditron_gemm_ar_two_shot     GEMM + AllReduce, tiles dealt to the ranks and broadcast
 *                               (paper, Appendix "GEMM All-Reduce")
 *
 * Conventions common to every entry point
 *   - "device" pointers are GPU global memory (or pinned host memory mapped into the GPU),
 *     "host" pointers are ordinary host memory read during the call.  All device buffers are
 *     owned by the caller; the library allocates no device memory and keeps no mutable state
 *     between calls (per-call options travel in ditron_tuning_t).
 *   - All device pointers must be 16-byte aligned.  Matrices are row-major and dense
 *     (leading dimension = number of columns).  bf16 is the upper half of an IEEE binary32;
 *     fp8 is OCP e4m3 (finite only, max 448).  The contraction length k must be a multiple
 *     of 8 (bf16) or 16 (fp8), n a multiple of 8.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and return; results are valid once the stream has been synchronised.
 *   - Signals.  `signals` is a caller-allocated int32 array of ditron_signal_words(world)
 *     words that the caller zero-fills once.  A flag "has arrived" when it equals `epoch`;
 *     pass a value different from every earlier call on the same buffer (e.g. 1, 2, 3, ...)
 *     so that no reset sits between calls.  Words beyond the flags are internal counters
 *     which every call leaves at zero.
 *     The epoch is a launch argument: a captured HIP graph would replay the same value, for which
 *     the flags of the previous replay already stand, so a graph must not replay these calls.
 *   - `status` is a device int32[DITRON_STATUS_WORDS], zero-filled by the caller.  Kernels
 *     never spin forever: a wait that exceeds the spin limit stores DITRON_ERR_TIMEOUT in
 *     status[0] (and the flag index in status[1]) and the work-group carries on, so the
 *     result is then undefined but the kernel terminates.
 *   - Who delivers the remote data is chosen by exactly one of three mode bits in `flags`:
 *     DITRON_EMULATE_PRODUCER (the call copies the peers' data itself and raises the flags, in the
 *     order the peers would), DITRON_EXTERNAL_PRODUCER (somebody else does, the kernels only wait)
 *     or DITRON_FLAGS_PRESET (everything is already in place: nothing is copied, no flag is
 *     looked at; the kernels alone, e.g. to time them).
 *   - `tuning` is a host pointer to per-call options, or NULL for the defaults.
 *   - Return value: DITRON_OK, or an error without any work having been enqueued.
 *     INVALID_ARG: null / misaligned pointer, non-positive size, rank outside [0, world),
 *     m not divisible by world, world > DITRON_MAX_WORLD, bad enum.  UNSUPPORTED: a
 *     size rule above is violated or the layout/dtype combination has no kernel.
 *     HIP: the launch failed.
 */
#ifndef DITRON_H
#define DITRON_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DITRON_OK = 0,
  DITRON_ERR_INVALID_ARG = 1,
  DITRON_ERR_UNSUPPORTED = 2,
  DITRON_ERR_WORKSPACE = 3,
  DITRON_ERR_HIP = 4,
  DITRON_ERR_TIMEOUT = 5
} ditron_status_t;

typedef enum { DITRON_BF16 = 0, DITRON_FP8_E4M3 = 1 } ditron_dtype_t;

/* Physical layout of the logical [k, n] right-hand matrix.  The bf16 AllGather-GEMM and
 * GEMM-ReduceScatter, GEMM + AllReduce and the MoE grouped GEMM take both; fp8 takes DITRON_B_NK only (UNSUPPORTED
 * otherwise). */
typedef enum {
  DITRON_B_KN = 0, /* stored [k, n], n contiguous */
  DITRON_B_NK = 1  /* stored [n, k], k contiguous: the weight layout of the paper's launchers */
} ditron_blayout_t;

enum {
  DITRON_EMULATE_PRODUCER = 1u,  /* the call itself copies the shards and raises the flags */
  DITRON_EXTERNAL_PRODUCER = 2u, /* somebody else fills the workspace and raises the flags   */
  DITRON_FLAGS_PRESET = 4u,      /* the remote data is resident: no copies, no flag waits    */
  DITRON_DUMP_SCHEDULE = 8u,     /* write the tile schedule to `schedule_out`                */
  DITRON_DUMP_TIMING = 16u,      /* ditron_ag_gemm: write per-work-group time stamps to `schedule_out`
                                  * instead (not together with DITRON_DUMP_SCHEDULE): the record of a GEMM
                                  * work-group, at the index its schedule record would have, is (start,
                                  * flag wait entered, flag wait left, end) in ticks of the GPU's constant
                                  * 100 MHz clock, low 31 bits: where a launch's time goes between waiting
                                  * for shards and computing (decode_variant 1 writes nothing) */
  DITRON_EPOCH_IN_MEMORY = 32u,  /* decode-shaped ditron_ag_gemm (decode_variant 0, 2, 3, 4): the `epoch`
                                  * argument is ignored; the call's epoch is 1 + the last word of `signals`,
                                  * and the kernel's last work-group to finish stores it there (the word
                                  * before it counts the finished work-groups and returns to zero).  The
                                  * same recorded launch can then be replayed, e.g. from a HIP graph: the
                                  * call makes no other host-side change between launches.  Calls with and
                                  * without this flag must not share a `signals` array.  Elsewhere:
                                  * DITRON_ERR_UNSUPPORTED */
};

/* Per-call options (host memory, read during the call).  A zero field means "default", so a
 * zero-filled struct and a NULL pointer are the same thing. */
typedef struct {
  int num_nodes;       /* nodes the `world` ranks are spread over (must divide world); 0 = 1.  With
                        * more than one node ditron_ag_gemm / ditron_gemm_rs visit the tile rows in
                        * the order of the paper's multi-node listings (see ditron_tile_row_order);
                        * a shape for which that order does not visit every tile row exactly once is
                        * refused with DITRON_ERR_UNSUPPORTED */
  unsigned spin_limit; /* flag polls per wait before DITRON_ERR_TIMEOUT; 0 = 1 << 20 (of the order
                        * of a second).  A tiny value lets a test exercise the time-out path without
                        * hanging a kernel */
  int decode_variant;  /* decode-shaped ditron_ag_gemm only, see there; 0 = the library's choice */
  int moe_route_groups; /* ditron_moe_ag_grouped_gemm only: work-groups that share the routing scan, 1..8;
                        * 0 = one per 4096 assignments.  The outputs do not depend on it */
  int reserved[4];     /* must be zero */
} ditron_tuning_t;

#define DITRON_MAX_WORLD 32
#define DITRON_STATUS_WORDS 4
#define DITRON_SCHEDULE_WORDS 4 /* int32 words per tile record in a schedule dump */
#define DITRON_TILE_CONFIG_WORDS 10
#define DITRON_MOE_ROUTE_SCRATCH_BYTES 266240u /* 8 work-groups x (32 x 256 + 128) int32 */

/* Number of int32 words the `signals` array of any entry point must have for `world`
 * ranks and `chunks` flags per rank (chunks = 1 except for ditron_gemm_rs): flags and arrival
 * counters per rank and per (rank, chunk), plus 16 words for the work-groups of the MoE routing. */
size_t ditron_signal_words(int world, int chunks);

/*
 * Tile rows across nodes.  Paper: Appendix "Swizzle", first listing (AllGather-GEMM) and second
 * listing (GEMM-ReduceScatter): with `nnodes` nodes of world/nnodes ranks, the gather order
 * visits the own node's tile rows first and inside a node starts at the own local rank; the
 * scatter order starts with the next node and the next local rank; a tile row shared by two
 * nodes is visited once: it belongs to whichever of the two nodes is visited later (gather: both
 * nodes' rows must have arrived) or earlier (scatter: it is computed as early as possible for both).
 * With one node these are the plain rotations.
 *
 * ditron_tile_row_order: evaluates the order on the host with the very function the kernels
 * use: out[t] (host int[ceil(m / block_m)]) = tile row visited at position t.  op 0 = gather
 * order, 1 = scatter order.  m = rows of the full matrix (a multiple of world).
 */
ditron_status_t ditron_tile_row_order(int op, int m, int block_m, int world, int nnodes, int rank, int* out);

/* Tile shape and ordering parameters the library will use for a problem, so that a test can
 * evaluate the schedule independently.  op: 0 = ag_gemm, 1 = gemm_rs, 2 = moe grouped gemm
 * (m = max_rows; the smallest BLOCK_M is reported and 0 for the column block: both are chosen per
 * call, see ditron_moe_tile_choice),
 * 3 = gemm_ar, 4 = ag_gemm with B stored [k, n] (bf16 problems with few 128 x 128 tiles and B stored
 * [n, k] use the 128 x 32 tile of the decode kernel, which the [k, n] layout does not).
 * out[0]=BLOCK_M out[1]=BLOCK_N out[2]=GROUP_SIZE_M out[3]=chiplets used by the work-group
 * remap (0 = no remap) out[4]=tiles per chiplet per block out[5]=number of tiles
 * (ag_gemm / gemm_rs) out[6]=threads per work-group out[7]=operand staging of the tile engine (0 = through
 * registers, 1 = global memory straight into LDS; op 1 and 3 report the choice for B stored [n, k])
 * out[8]=work-groups that share the contraction of one output tile (decode-shaped ag_gemm; else 1): a
 * schedule dump then holds that many identical records per tile, tile after tile.  out[9]=0.
 * `tuning`: only decode_variant matters. */
ditron_status_t ditron_tile_config(int op, int m, int n, int k, int dtype, const ditron_tuning_t* tuning,
                                   int out[DITRON_TILE_CONFIG_WORDS]);

/*
 * Sizes of the buffers the launchers' contexts own in the paper (`ag_gemm(a, b, ctx)`: the
 * symmetric workspace that receives the gathered A; the MoE launcher: the gathered tokens).
 * Bytes of the `workspace` argument of ditron_ag_gemm (the gathered [world*m_per_rank, k] in `dtype`;
 * for decode-shaped problems, whose contraction is split over several work-groups, followed at the next
 * multiple of 256 bytes by the fp32 partial tiles) and of ditron_moe_ag_grouped_gemm
 * ([world*tokens_per_rank, hidden] bf16, followed at the next multiple of 256 bytes by
 * DITRON_MOE_ROUTE_SCRATCH_BYTES through which the routing work-groups exchange their histograms;
 * that part needs no initialisation); 0 for invalid arguments.
 * The other caller-sized arrays have closed forms given with their arguments (signals:
 * ditron_signal_words; tile_records: ditron_moe_max_tiles).
 */
size_t ditron_ag_gemm_workspace_bytes(int m_per_rank, int n, int k, int world, int dtype, int b_layout,
                                      const ditron_tuning_t* tuning);
size_t ditron_moe_workspace_bytes(int tokens_per_rank, int hidden, int world);

/*
 * The tile schedule of a call, evaluated on the host with the functions the kernels use (paper: the
 * index arithmetic at the top of `kernel_consumer_gemm` and `kernel_gemm_rs_producer`: grouped order,
 * rank rotation, wait set / segment span).  op: 0 = ditron_ag_gemm, 1 = ditron_gemm_rs,
 * 3 = ditron_gemm_ar (m, n, k as passed to those calls; for op 0 m = world*m_per_rank).
 * out (host int32[DITRON_SCHEDULE_WORDS * capacity]) receives one record per GEMM work-group, in
 * work-group order: (pid_m, pid_n, first, last) with first..last the shards waited for (op 0) or the
 * segments touched (op 1); op 3: the record of position t of the tile order is (pid_m, pid_n, 0, 0).
 * *count receives the number of records.  DITRON_ERR_WORKSPACE (and *count set) if capacity is too
 * small.  Identical, word for word, to what DITRON_DUMP_SCHEDULE makes the kernels write (op 3: to its
 * first two words).
 */
ditron_status_t ditron_schedule_dump(int op, int m, int n, int k, int world, int rank, int dtype, int b_layout,
                                     const ditron_tuning_t* tuning, int32_t* out, int capacity, int* count);

/*
 * AllGather-GEMM:  C[world*m_per_rank, n] = concat_s(A_s) . B       (fp32 accumulate)
 *
 * Paper: host launcher `ag_gemm`, producer `cp_engine_producer_all_gather_full_mesh_pull`
 * and consumer `kernel_consumer_gemm` of Appendix "AllGather GEMM".  Shard s lands at rows
 * [s*m_per_rank, (s+1)*m_per_rank) of `workspace` and flag s is raised after it; a tile
 * whose rows touch shards rank_beg..rank_end waits for exactly those flags; tile rows are
 * visited starting at the rank's own shard.
 *
 *  a_shards      host array of `world` device pointers, each [m_per_rank, k] in `dtype`
 *                (EMULATE_PRODUCER; ignored with EXTERNAL_PRODUCER)
 *  b, b_layout   device, logical [k, n] in `dtype`, layout ditron_blayout_t
 *  c             device out, [world*m_per_rank, n] bf16
 *  a_scales      device float[world] (fp8: one scale per shard) or NULL
 *  b_scales      device float[n]     (fp8: one scale per output column) or NULL
 *                fp8 result is (sum_k a*b) * a_scales[row / m_per_rank] * b_scales[col]
 *  workspace     device, ditron_ag_gemm_workspace_bytes(...) bytes; starts with the gathered A,
 *                [world*m_per_rank, k] in `dtype` (written by the producer, read by the GEMM).
 *                For decode-shaped problems the partial tiles behind it are exchanged flag-in-data:
 *                every 8-byte word carries the call's epoch, so like `signals` the workspace must be
 *                zero-filled once before its first use, and the epoch must be nonzero and must not
 *                repeat an earlier call's on the same workspace
 *  signals       device int32[ditron_signal_words(world, 1)]; flag s is word s
 *  status        device int32[DITRON_STATUS_WORDS]
 *  schedule_out  device int32[4 * tiles] or NULL; with DITRON_DUMP_SCHEDULE the GEMM
 *                work-group with index w writes (pid_m, pid_n, rank_beg, rank_end) at 4*w
 *  arrival_order host int[world] or NULL: the order in which the emulated producer delivers
 *                shards; NULL = rank, rank+1, ... (mod world) as in the paper's producer
 *  tuning->decode_variant (fp8, and bf16 problems of at most 128 tiles of 128 x 128 with B stored
 *                [n, k]; the latency variants of the paper's Section "Kernel library"): 0 = library's
 *                choice; 1 = 128 x 32 tiles over the whole contraction; 2 = 128 x 128 tiles, the
 *                contraction split over up to 8 work-groups whose fp32 partials are summed in split
 *                order by the last to finish; 3 = the same with 128 x 64 tiles; 4 = 16-row tiles,
 *                one shard's rows at the decode shape, each waiting for its own shard only
 */
ditron_status_t ditron_ag_gemm(const void* const* a_shards, const void* b, int b_layout, void* c,
                               const float* a_scales, const float* b_scales, void* workspace,
                               int32_t* signals, int32_t* status, int32_t* schedule_out,
                               const int* arrival_order, int m_per_rank, int n, int k, int world,
                               int rank, int dtype, int32_t epoch, unsigned flags, const ditron_tuning_t* tuning, void* stream);

/*
 * ditron_ag_gemm for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The scratch of ditron_ag_gemm (the `workspace` that
 * receives the gathered A and the `signals` words) comes from a fixed array inside the library's device
 * image (DITRON_STATIC_WORKSPACE_BYTES + 4 KiB, one copy per GPU the library has been called on, held
 * until the process ends); the call allocates nothing and frees nothing.  Always in
 * DITRON_EMULATE_PRODUCER mode (nobody else can reach the workspace); arguments as for ditron_ag_gemm.
 * DITRON_ERR_WORKSPACE if ditron_ag_gemm_workspace_bytes(m_per_rank, n, k, world, dtype, b_layout, tuning) exceeds
 * DITRON_STATIC_WORKSPACE_BYTES, before anything is enqueued.  The signal words are cleared on the
 * stream at the start of every call (by a small kernel, so the call may be captured), and the call's
 * epoch comes from a per-GPU call count kept on the host (a captured graph replays the epoch it was
 * captured with: replay a captured call of a decode-shaped problem at most once per capture).  Every call on
 * a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race.
 */
#define DITRON_STATIC_WORKSPACE_BYTES (32u << 20)
ditron_status_t ditron_ag_gemm_static(const void* const* a_shards, const void* b, int b_layout, void* c,
                                      const float* a_scales, const float* b_scales, int32_t* status,
                                      const int* arrival_order, int m_per_rank, int n, int k, int world,
                                      int rank, int dtype, const ditron_tuning_t* tuning, void* stream);

/*
 * GEMM-ReduceScatter:  out[m/world, n] = rows_rank( sum_s P_s ),  P_rank = A . B computed here.
 *
 * Paper: `gemm_rs_op`, `kernel_gemm_rs_producer` and the reduce-scatter launchers of Appendix
 * "GEMM Reduce-Scatter".  The GEMM visits tile rows starting at the segment of rank+1 and
 * ending with the rank's own; every tile adds one to the counter of each segment it touches
 * and the tile that completes a segment raises that segment's flag.  The blocks the peers
 * would push into this rank's scatter buffer are copied there (peer by peer, in the order
 * rank-1, rank-2, ..., unless `arrival_order` says otherwise) with one flag per
 * (peer, row chunk).  The reduction adds the `world` blocks in fp32, in slot order, and
 * rounds once to bf16; a row chunk is reduced once its `world` flags are up.
 *
 *  a             device [m, k_local] bf16
 *  b, b_layout   device, logical [k_local, n] bf16
 *  gemm_out      device out [m, n] bf16: this rank's partial product
 *  peer_partials host array of `world` device pointers; entry s != rank is the [m/world, n]
 *                bf16 block that rank s contributes to this rank (entry `rank` is ignored:
 *                the own block is rows rank*m/world.. of gemm_out)
 *  scatter_buf   device [world, m/world, n] bf16: the destination slots (slot `rank` unused)
 *  out           device out [m/world, n] bf16
 *  signals       device int32[ditron_signal_words(world, chunks_per_slot)]:
 *                words [0, world) are the GEMM's segment flags; the arrival flag of
 *                (peer s, row chunk c) is word 2*world + s*chunks_per_slot + c
 *  schedule_out  with DITRON_DUMP_SCHEDULE: (pid_m, pid_n, segment_start, segment_end) per
 *                GEMM work-group
 *  arrival_order host int[world-1] (peers in delivery order) or NULL
 *  chunks_per_slot  row chunks per slot (>= 1, must divide m/world)
 */
ditron_status_t ditron_gemm_rs(const void* a, const void* b, int b_layout, void* gemm_out,
                               const void* const* peer_partials, void* scatter_buf, void* out,
                               int32_t* signals, int32_t* status, int32_t* schedule_out,
                               const int* arrival_order, int m, int n, int k_local, int world,
                               int rank, int chunks_per_slot, int32_t epoch, unsigned flags,
                               const ditron_tuning_t* tuning, void* stream);

/*
 * GEMM-ReduceScatter with the scatter fused into the GEMM's stores.  Paper: the FUSE_SCATTER branch of
 * `kernel_gemm_rs_producer` and of `gemm_rs_op` (Appendix "GEMM Reduce-Scatter"): instead of writing
 * its partial product to a local [m, n] buffer, a tile stores the rows of segment d directly into
 * rank d's buffer, row m landing at row rank*(m/world) + m % (m/world), i.e. in slot `rank` of
 * that rank's [world, m/world, n] buffer; the reduction then sums the `world` slots of the local
 * buffer.  Everything else (tile order, segment counters and flags, emulated arrival of the
 * peers' blocks into the local slots, gated reduction) is as in ditron_gemm_rs.
 *
 *  scatter_dsts  host array of `world` device pointers, each a [world, m/world, n] bf16 buffer:
 *                entry d stands for the buffer of rank d (on one GPU: any distinct device
 *                buffers); entry `rank` is this rank's own buffer, the one the peers' blocks
 *                arrive in and the reduction reads.  Only slot `rank` of the other entries is
 *                written.
 *  other arguments as for ditron_gemm_rs (there is no gemm_out).
 */
ditron_status_t ditron_gemm_rs_fuse_scatter(const void* a, const void* b, int b_layout,
                                            void* const* scatter_dsts, const void* const* peer_partials,
                                            void* out, int32_t* signals, int32_t* status,
                                            int32_t* schedule_out, const int* arrival_order, int m,
                                            int n, int k_local, int world, int rank,
                                            int chunks_per_slot, int32_t epoch, unsigned flags,
                                            const ditron_tuning_t* tuning, void* stream);

/*
 * GEMM + AllReduce, one-shot:  out[m, n] = sum_s P_s,  P_rank = A . B computed here.
 *
 * Paper: `gemm_allreduce_op`, `kernel_persistent_gemm_notify` and `consumer_all_reduce_kernel`
 * of Appendix "GEMM All-Reduce", the branch that reduces every tile on every rank.  The tiles
 * of P_rank are computed in the grouped order, each stored into `gemm_out` (the buffer the
 * peers read) and announced by that tile's flag.  The consumer takes the tiles in the same
 * order, waits for the tile's flag of every rank, adds the `world` published tiles in fp32 in
 * rank order (the paper reduces through the switch; here in software) and rounds once to bf16.
 * GEMM tiles and consumer work-groups share one launch: some consumers follow the first
 * chip-wide round of tiles and reduce finished tiles while later rounds are computed, the rest
 * follow the last tile.
 *
 *  a             device [m, k_local] bf16
 *  b, b_layout   device, logical [k_local, n] bf16
 *  gemm_out      device out [m, n] bf16: this rank's partial product
 *  peer_partials host array of `world` device pointers; entry s != rank is rank s's published
 *                partial [m, n] bf16, read in place (entry `rank` is ignored); NULL if world = 1.
 *                With DITRON_EXTERNAL_PRODUCER a tile of it must be complete before its flag
 *                is raised.
 *  out           device out [m, n] bf16, distinct from every partial
 *  signals       device int32[ditron_signal_words(world, tiles)], tiles as reported by
 *                ditron_tile_config(3, ...): the flag of (rank s, tile (pid_m, pid_n)) is word
 *                2*world + s*tiles + pid_m*ceil(n / BLOCK_N) + pid_n; words 0 and 1 are the
 *                consumer's queue counters, left at zero by every call
 *  schedule_out  device int32[4 * tiles] or NULL; with DITRON_DUMP_SCHEDULE the record of
 *                position t of the tile order is (pid_m, pid_n, index of the tile's work-group
 *                in the launch with the emulated peers not counted, 0)
 *  DITRON_EMULATE_PRODUCER: the call raises the peers' tile flags itself, in tile order.
 *  m need not be a multiple of world.
 */
ditron_status_t ditron_gemm_ar(const void* a, const void* b, int b_layout, void* gemm_out,
                               const void* const* peer_partials, void* out, int32_t* signals,
                               int32_t* status, int32_t* schedule_out, int m, int n, int k_local,
                               int world, int rank, int32_t epoch, unsigned flags, const ditron_tuning_t* tuning, void* stream);

/*
 * GEMM + AllReduce, two-shot: the default branch of the same listings (USE_MULTIMEM_ST).  The tiles
 * are dealt to the ranks; a rank reduces only the tiles it owns (waiting for their flags from every
 * rank) and stores each reduced tile into every rank's output buffer, and the other tiles of its own
 * output arrive from their owners; the call ends once every peer has signalled that its tiles have
 * been broadcast.  The paper deals blocks of NUM_COMM_SMS consecutive tile ids round-robin; here
 * position q of the GEMM's tile order belongs to rank q % world.  The paper broadcasts through the
 * switch (`multimem.st`); here with one store per destination.
 *
 *  out_dsts      host array of `world` device pointers [m, n] bf16: entry d stands for the output
 *                buffer of rank d (on one GPU: any distinct device buffers); entry `rank` is this
 *                rank's output, complete when the call returns.  Of the other entries only the
 *                tiles this rank owns are written.
 *  peer_reduced  DITRON_EMULATE_PRODUCER: host array of `world` device pointers [m, n] bf16, entry
 *                s != rank holding what rank s broadcasts (only the tiles it owns are read); the
 *                emulated peers copy those tiles into this rank's output and then raise the flags
 *                below.  Ignored with DITRON_EXTERNAL_PRODUCER.
 *  signals       as for ditron_gemm_ar, plus word 2*world + world*tiles + s: rank s has broadcast
 *                all its tiles (raised by the peers; word 2 is an internal counter left at zero)
 *  other arguments as for ditron_gemm_ar.
 */
ditron_status_t ditron_gemm_ar_two_shot(const void* a, const void* b, int b_layout, void* gemm_out,
                                        const void* const* peer_partials, void* const* out_dsts,
                                        const void* const* peer_reduced, int32_t* signals,
                                        int32_t* status, int32_t* schedule_out, int m, int n,
                                        int k_local, int world, int rank, int32_t epoch,
                                        unsigned flags, const ditron_tuning_t* tuning, void* stream);

/*
 * The reduction step of GEMM-ReduceScatter on its own: out = bf16( sum_s fp32(slots[s]) ),
 * slot order 0..world-1.  slots: host array of `world` device pointers [rows, n] bf16.
 * `signals` may be NULL (no gating); otherwise word s*chunks + c gates row chunk c of slot s.
 */
ditron_status_t ditron_reduce_slots(const void* const* slots, void* out, const int32_t* signals,
                                    int32_t* status, int rows, int n, int world, int chunks,
                                    int32_t epoch, const ditron_tuning_t* tuning, void* stream);

/*
 * MoE: route -> (all-gathered) token rows grouped by expert -> grouped GEMM.
 *
 * Paper: "ag_group_gemm" in the kernel list; tile ordering from
 * `threadblock_swizzle_ag_moe_kernel`.  Token t = s*tokens_per_rank + i lives in shard s;
 * assignment f = t*top_k + j goes to expert topk_ids[f].  For the local experts
 * [expert_begin, expert_begin + num_local_experts):
 *   counts[s*num_experts + e]  assignments of shard s to expert e (all experts)
 *   expert_offsets[j]          exclusive prefix sum of the local experts' totals; [E_l] = R
 *   gather_idx[offset_j + q]   q-th smallest f routed to local expert j
 *   y[p, :] = X[gather_idx[p] / top_k, :] . W_j   for p in the rows of expert j, fp32 accumulate
 * Row tiles are ordered by (expert, arrival stage of the last shard they need) and each
 * waits for the shard flags it needs.
 *
 *  x_shards      host array of `world` device pointers [tokens_per_rank, hidden] bf16
 *  topk_ids      device int32 [world*tokens_per_rank, top_k]
 *  w, w_layout   device, per expert logical [hidden, inter] bf16, experts contiguous;
 *                layout as ditron_blayout_t (DITRON_B_NK = [E_l, inter, hidden], DITRON_B_KN =
 *                [E_l, hidden, inter])
 *  y             device out [max_rows, inter] bf16; rows >= R are not written
 *  counts        device out int32 [world * num_experts]
 *  expert_offsets device out int32 [num_local_experts + 1]
 *  gather_idx    device out int32 [max_rows]
 *  tile_records  device out int32 [1 + 5*max_tiles], max_tiles =
 *                ditron_moe_max_tiles(max_rows, num_local_experts): word 0 = ntiles, then
 *                (expert_id, tiled_m, segment_start, segment_end) per tile in execution
 *                order (expert_id counted from expert_begin, tiled_m = index of the tile in
 *                the unsorted per-expert order); the last max_tiles words are internal
 *                (first output row of each tile)
 *  workspace     device, ditron_moe_workspace_bytes(tokens_per_rank, hidden, world) bytes: the gathered
 *                tokens [world*tokens_per_rank, hidden] bf16, then scratch of the routing scan
 *  signals       device int32[ditron_signal_words(world, 1)]: shard flags and arrival counters in
 *                the first 2*world words; the last 16 words are the routing work-groups' flags
 *  The routing scan is shared by tuning->moe_route_groups work-groups (contiguous ranges of the flat
 *  assignment index; they exchange their histograms through the scratch, one bounded wait each).
 *  If R exceeds max_rows, status[0] = DITRON_ERR_WORKSPACE, status[2] = R and no GEMM tile
 *  runs.  An expert id outside [0, num_experts) is an error, not a dropped assignment:
 *  status[0] = DITRON_ERR_INVALID_ARG, status[1] = the smallest flat index f holding such an id,
 *  and no GEMM tile runs (counts then holds the in-range ids only; expert_offsets and gather_idx
 *  are not written).  Limits: num_experts <= 256, num_local_experts <= 64, max_tiles <= 4096.
 */
ditron_status_t ditron_moe_ag_grouped_gemm(const void* const* x_shards, const int32_t* topk_ids,
                                           const void* w, int w_layout, void* y, int32_t* counts,
                                           int32_t* expert_offsets, int32_t* gather_idx,
                                           int32_t* tile_records, void* workspace,
                                           int32_t* signals, int32_t* status,
                                           const int* arrival_order, int tokens_per_rank,
                                           int hidden, int inter, int num_experts, int top_k,
                                           int expert_begin, int num_local_experts, int max_rows,
                                           int world, int rank, int32_t epoch, unsigned flags,
                                           const ditron_tuning_t* tuning, void* stream);

/*
 * MoE down-projection + ReduceScatter:  out[tokens_per_rank, hidden] = rows_rank( sum_s z_s ),
 *   z_rank[t, :] = sum_j gate[t, j] * ( h[pos(t*top_k + j), :] . W2_expert(t, j) )   computed here.
 *
 * Paper: the workload "MoE+ReduceScatter" of the evaluation (tensor-parallel placement: every rank holds
 * its slice of the intermediate dimension of every expert); the paper prints its shape, not a listing, so
 * the steps are the plain ones.  The activations are grouped by expert already (row p belongs to the
 * assignment gather_idx[p]: the output order of ditron_moe_ag_grouped_gemm), the grouped GEMM multiplies
 * each expert's rows by its down-projection, the combine adds a token's top_k rows (fp32 fused multiply-add
 * in the order j = 0..top_k-1, one rounding to bf16; an assignment whose expert is not on the rank adds
 * nothing), and the reduce-scatter is that of ditron_gemm_rs: the peers' blocks arrive in the scatter
 * buffer (emulated: copied there in the order rank-1, rank-2, ...), the `world` slots are added in fp32 in
 * slot order and rounded once.
 *
 *  h             device [R, inter] bf16, R = expert_offsets[num_local_experts] <= max_rows
 *  w, w_layout   device, per expert logical [inter, hidden] bf16 (DITRON_B_NK = [E_l, hidden, inter],
 *                DITRON_B_KN = [E_l, inter, hidden])
 *  topk_weights  device float[world*tokens_per_rank*top_k] or NULL (all ones)
 *  gather_idx, expert_offsets   device, as written by ditron_moe_ag_grouped_gemm
 *  y             device scratch [max_rows, hidden] bf16: the grouped GEMM's output
 *  inverse_idx   device scratch int32[world*tokens_per_rank*top_k]
 *  tile_records  device scratch int32[1 + 5*ditron_moe_max_tiles(max_rows, num_local_experts)]
 *  combined      device out [world*tokens_per_rank, hidden] bf16: this rank's partial z_rank
 *  peer_partials host array of `world` device pointers; entry s != rank is the [tokens_per_rank, hidden]
 *                bf16 block rank s contributes to this rank (EMULATE_PRODUCER)
 *  scatter_buf   device [world, tokens_per_rank, hidden] bf16 (slot `rank` unused)
 *  out           device out [tokens_per_rank, hidden] bf16
 *  signals       device int32[ditron_signal_words(world, chunks_per_slot)], laid out as for ditron_gemm_rs:
 *                the arrival flag of (slot s, row chunk c) is word 2*world + s*chunks_per_slot + c; the
 *                own slot's flags are raised by the combine
 *  If R exceeds max_rows: status[0] = DITRON_ERR_WORKSPACE, status[2] = R, and `out` is undefined.
 */
ditron_status_t ditron_moe_grouped_gemm_rs(const void* h, const void* w, int w_layout, const float* topk_weights,
                                           const int32_t* gather_idx, const int32_t* expert_offsets, void* y,
                                           int32_t* inverse_idx, int32_t* tile_records, void* combined,
                                           const void* const* peer_partials, void* scatter_buf, void* out,
                                           int32_t* signals, int32_t* status, const int* arrival_order,
                                           int tokens_per_rank, int hidden, int inter, int num_experts, int top_k,
                                           int num_local_experts, int max_rows, int world, int rank,
                                           int chunks_per_slot, int32_t epoch, unsigned flags,
                                           const ditron_tuning_t* tuning, void* stream);

/* Tile of the grouped GEMM for a call with these sizes (total_tokens = world * tokens_per_rank):
 * out[0] = BLOCK_M (128, or 256 when the experts are large), out[1] = BLOCK_N.  The tile schedule
 * in tile_records is cut with this BLOCK_M. */
ditron_status_t ditron_moe_tile_choice(int total_tokens, int top_k, int num_experts,
                                       int num_local_experts, int inter, int out[2]);

/* Upper bound on the number of row tiles of the grouped GEMM. */
int ditron_moe_max_tiles(int max_rows, int num_local_experts);

/*
 * Test / integration helper: an external producer.  Copies n chunks (dst[i] <- src[i],
 * bytes[i] bytes, multiples of 16) in the given order on `stream`, raising
 * signals[flag_index[i]] = epoch after each, optionally idling `delay_cycles` GPU clock
 * ticks before each chunk.  All array arguments are host arrays of length n (n <= 64).
 */
ditron_status_t ditron_publish_chunks(void* const* dst, const void* const* src,
                                      const size_t* bytes, const int* flag_index,
                                      int32_t* signals, int n, int32_t epoch,
                                      unsigned delay_cycles, void* stream);

const char* ditron_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DITRON_H */
