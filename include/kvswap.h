/*
 * kvswap.h - C ABI of the MI355X KV-cache context-switch library.
 *
 * The library moves a preempted request's paged KV cache from GPU HBM to
 * pinned host memory and back (FastSwitch, arXiv 2411.18424: Section 2.1
 * preemption by swapping, Section 3.1 block groups, Section 3.2 asynchronous
 * swapping, Section 3.3 reuse of the CPU copy).  The data path is
 *
 *   swap-out: gather kernel (scattered pool chunks -> contiguous device
 *             staging) -> large pinned device-to-host copies
 *   swap-in : large pinned host-to-device copies -> scatter kernel (staging ->
 *             freshly allocated pool chunks)
 *
 * on dedicated HIP streams ordered by events, so that both directions overlap
 * each other and the caller's compute.
 *
 * Conventions
 *  - Every function returns 0 (KV_OK) or a negative kv_status_t.  No function
 *    throws or aborts.  All argument validation happens before anything is
 *    enqueued: a call that returns an error has had no effect.  (KV_EHIP is the
 *    exception: a HIP runtime call that fails in the middle of a call can leave it
 *    half enqueued; destroy the pool then.)
 *  - All pointers are HOST pointers unless a comment says "device pointer".
 *  - The caller owns every array it passes; the library has consumed it when
 *    the call returns.  The library owns the pool object, the pinned host
 *    arena, its streams and events, and (unless supplied) the staging ring.
 *  - Block ids are int32 in [0, n_gpu_blocks).  Request ids are caller-chosen
 *    int64 values.
 *  - swap_* calls are asynchronous: they enqueue work and return.  Use
 *    kv_wait / kv_query / kv_stream_wait to observe completion.
 *  - A kv_pool_t may be used from several host threads (one internal lock).
 *
 * Layouts (bytes; all elements are opaque, NaN/Inf payloads survive bit-exact)
 *  - chunk  C = block_size * n_kv_heads * head_dim * elt_bytes, a multiple of 16
 *  - GPU pool:   pool[p][b][C],  plane p = 2*layer + kv (kv 0 = K, 1 = V),
 *                P = 2*n_layers planes, b in [0, n_gpu_blocks)
 *  - host image of a request with n logical blocks: image[j][p][C], j < n
 *                (one block record R = P*C bytes per logical block)
 */
#ifndef KVSWAP_H
#define KVSWAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KV_OK          =  0,
  KV_EINVAL      = -1, /* bad argument: id out of range, duplicate id, length mismatch, bad shape */
  KV_ENOMEM_GPU  = -2, /* no free GPU blocks / device allocation failed */
  KV_ENOMEM_HOST = -3, /* pinned host arena exhausted */
  KV_ENOENT      = -4, /* request has no (valid) host copy */
  KV_EBUSY       = -5, /* object still in use */
  KV_EHIP        = -6, /* a HIP runtime call failed; see kv_last_error() */
  KV_ENODEV      = -7  /* operation needs a device but the pool is plan-only */
} kv_status_t;

/* flags for kv_pool_config_t.flags */
#define KV_FLAG_PLAN_ONLY        1u /* no HIP call is ever made and no byte moves: only validation,
                                       allocator and reuse-map bookkeeping run (host-logic tests) */
#define KV_FLAG_PROFILE          2u /* time every kernel launch and copy with HIP events (kv_profile_*) */
#define KV_FLAG_ORDER_COMPUTE    4u /* order swaps after work already enqueued on compute_stream */
#define KV_FLAG_MAPPED_SWAP_IN  16u /* swap-in reads the pinned host image directly from a small scatter
                                       kernel (no staging, no copy engine): lower latency, and the cost no
                                       longer depends on how fragmented the moved set is */
#define KV_FLAG_MAPPED_SWAP_OUT 64u /* swap-outs that move at most mapped_out_max_blocks blocks are done by
                                       one kernel that stores the records straight into the pinned image
                                       (no staging, no copy): lowest latency for small requests.  Stores to
                                       host memory slow HBM-bound kernels running beside them, so larger
                                       swap-outs keep using the copy engines */
#define KV_FLAG_HOST_EVICT      32u /* when the host arena is full, reclaim the host copies of other requests
                                       (Section 3.3: contamination by higher-priority requests): lowest
                                       priority first, least recently used first, never from a request of
                                       higher priority than the caller's or with work in flight.  Room held
                                       in reserve goes first, then the records of the victim's last logical
                                       blocks, whose host_valid bits are cleared */
#define KV_FLAG_FOUR_STREAMS     8u /* separate streams for kernels and copies of each direction (default:
                                       one stream per direction, which needs fewer hardware queues): the
                                       copies of a piece of a swap-out start right behind its gather and the
                                       later gathers run under them; scatters run under the next copies.  Only
                                       where the process has hardware queues to spare (HIP's default is 4
                                       per process, GPU_MAX_HW_QUEUES): streams that share a queue with the
                                       application's compute stream wait behind its kernels */
#define KV_FLAG_SCATTER_STREAM 128u /* three streams: the scatter kernels get a stream of their own, so the
                                       scatter of a piece runs under the next piece's host-to-device copy */

#define KV_FLAG_NO_DEFER_COPIES 512u /* every swap-out's device-to-host copies are enqueued inside the swap-out
                                       call and wait for their gathers on the device.  Default (flag off): a
                                       swap-out that moves defer_min_bytes or more has its copies handed to the
                                       runtime only when the gathers they follow have finished - a thread of the
                                       pool waits for each piece's gathers on the host, then enqueues its copies
                                       (Section 3.2's control of dispatch order, made inside the library).
                                       Copies enqueued at once wait inside a copy engine's queue, where a
                                       host-to-device copy of another request can end up behind them: a swap-in
                                       issued right after a swap-out then finishes late, and callers have to
                                       issue the swap-in first.  With the copies held back the order of the two
                                       calls does not matter.  The swap-out call returns when its gathers are
                                       enqueued, as always; kv_query reports it unfinished and the waits block
                                       until the copies are done; a swap-in or swap-out of the same request,
                                       and a swap-out that does not fit the out ring beside the held-back ones,
                                       first wait on the host for the hand-over.  Costs a few
                                       microseconds per swap-out. */
#define KV_FLAG_SECOND_LANE   1024u /* a held-back swap-out (see above) of many scattered records of 1 to 8 MiB
                                       sends them as plain copies, every other one on the host-to-device stream,
                                       while no swap-in is in flight: that stream's copy engine would otherwise be
                                       idle, and two engines overlap the pause each makes between two copies
                                       (Section 3.3's increments with contaminated blocks: 50.8 -> 52-53 GB/s).
                                       A swap-in issued meanwhile queues behind those copies (at most 256 MiB of
                                       them).  Off by default: which copy engine a stream uses is the runtime's
                                       choice; the library arranges its calls so that the two streams got different
                                       ones in every process measured, and loses 10 % where they do not */
#define KV_FLAG_NO_LAUNCH_EVENTS 2048u /* the gather and scatter launches of a swap of defer_min_bytes or more are
                                        plain launches.  Default (flag off): they carry begin and end events of
                                        their own, as under KV_FLAG_PROFILE, although nobody reads them: with
                                        plain launches a swap-out and a swap-in that run at the same time shared
                                        the link badly in some call patterns (one after the other instead of side
                                        by side; a swap-out issued before the step's swap-in cost it 7 ms at the
                                        median and 30 ms at the 99th percentile).  For comparison */
#define KV_FLAG_NO_STRIDED_COPIES 256u /* one copy per run of adjacent host records, never a 2-D copy over
                                       several equal runs a constant stride apart (for comparison) */

typedef struct kv_pool kv_pool_t;

typedef struct {
  int32_t n_layers, n_kv_heads, head_dim, block_size, elt_bytes;
  int32_t flags;            /* KV_FLAG_* */
  int64_t n_gpu_blocks;     /* N */
  void*   gpu_base;         /* device pointer, >= P*N*C bytes, 16-byte aligned; caller-owned */
  int64_t host_bytes;       /* capacity of the pinned host arena (library allocates it) */
  void*   staging_base;     /* device pointer to staging_out_bytes + staging_in_bytes of staging
                               memory, or NULL: library allocates (then both sizes may be 0) */
  int64_t staging_out_bytes;/* swap-out staging ring; 0 = default min(4 GiB, pool/4).  A swap-out
                               call that fits is packed completely before its copies start */
  int64_t staging_in_bytes; /* swap-in staging ring; 0 = default min(1 GiB, pool/8) */
  int64_t max_piece_bytes;  /* most bytes one piece (pack launches + their copies) carries;
                               0 = default.  Always <= half a ring and >= one block record */
  int64_t copy_chunk_bytes; /* a host<->device copy is issued in pieces of at most this many
                               bytes so other streams' copies can interleave (Section 3.2,
                               dispatch-order control); 0 = default 256 MiB */
  void*   compute_stream;   /* hipStream_t of the caller's inference work (used with
                               KV_FLAG_ORDER_COMPUTE) */
  int32_t host_slack_blocks;/* room reserved after each new host image for the next turn's
                               increment (Section 3.3 adjacent preallocation); <0 = default 32 */
  int32_t gather_grid;      /* workgroups per launch of the persistent pack variant; 0 = default */
  int32_t tile_unroll;      /* 16-byte vectors per lane per tile (1,2,4,8); 0 = from chunk size */
  int32_t pack_variant;     /* 0 = one tile per workgroup, 256 lanes, tiles in XCD-aware order for
                               launches of 64 blocks or more (default); 2 = the same kernel always
                               in plain 3-D grid order; 1 = persistent
                               grid-stride workgroups with the block table in LDS;
                               3 = tile kernel with 1024 lanes; 4..7 = as 0 with the store cache
                               policy forced (bit 0: gather, bit 1: scatter stores at agent scope),
                               for comparison */
  int32_t mapped_in_grid;   /* workgroups of the mapped swap-in / swap-out kernels; 0 = default 64 */
  int32_t mapped_out_max_blocks; /* with KV_FLAG_MAPPED_SWAP_OUT: largest moved set that takes the
                               mapped path; 0 = every swap-out; < 0 is KV_EINVAL */
  int64_t defer_min_bytes;  /* smallest swap-out (bytes moved) whose copies are held back until its
                               gathers have finished (see KV_FLAG_NO_DEFER_COPIES); 0 = default
                               16 MiB, 1 = every swap-out; < 0 is KV_EINVAL */
} kv_pool_config_t;

/* Section 3.1 (KV pool + block groups).  Creates the pool object: pinned host arena,
 * staging rings, side streams, event pool, allocator with all N blocks free.
 * *out is written only on success. */
int32_t kv_pool_create(const kv_pool_config_t* cfg, kv_pool_t** out);
/* Waits for the library's own in-flight work (its streams, not the caller's), then frees
 * everything the library owns. */
int32_t kv_pool_destroy(kv_pool_t* pool);

/* Section 3.1, Dynamic Block Group allocation.  Returns n_blocks physical ids in
 * out_blocks[n_blocks] (caller-allocated), in as few maximal contiguous runs as the free
 * lists allow: the best-fitting free run when one holds the whole request, else the longest
 * free runs first.  min_run (>= 0; 0 and 1 mean no preference) is the block-group size the
 * caller is aiming for: the last piece of a request that had to be split is carved from the
 * best-fitting free run of at least min_run blocks when there is one, so free runs shorter
 * than min_run are touched only when every longer run is used up.  req is a label for the
 * caller's bookkeeping (ownership is not tracked per request).
 * *out_n_runs (may be NULL) receives the number of maximal runs.  Freed blocks that an
 * unfinished gather still reads or an unfinished scatter still writes are never handed out
 * (Section 3.2, KV cache conflict): if they are needed the call waits for exactly that work.  KV_ENOMEM_GPU if fewer than
 * n_blocks are free; nothing is allocated then. */
int32_t alloc_block_group(kv_pool_t* pool, int64_t req, int32_t n_blocks, int32_t min_run,
                          int32_t* out_blocks, int32_t* out_n_runs);
/* Returns blocks to the free lists (adjacent free runs merge).  Blocks named by a swap_out
 * whose gather, or by a swap_in whose scatter, has not finished stay unavailable until it
 * has: the allocator never hands out a block that work of this library still reads or
 * writes.  (Accesses from the caller's own streams are the caller's to order, with
 * kv_stream_wait and KV_FLAG_ORDER_COMPUTE.)  KV_EINVAL if any block is out of range,
 * repeated, or not currently allocated (then nothing is freed). */
int32_t free_block_group(kv_pool_t* pool, int64_t req, const int32_t* blocks, int32_t n_blocks);
/* Number of blocks currently free (including those waiting for a gather to finish). */
int32_t kv_free_blocks(kv_pool_t* pool, int64_t* out_free, int64_t* out_largest_run);

/* Section 3.1, Dynamic Block Group Manager: requests that grow.  A request owns block groups
 * (contiguous runs); its newest group is the active one and carries a reserved tail the request
 * grows into.  kv_bg_append gives req n_blocks more blocks (a request is created by its first
 * append): from the active group's tail, else by growing that group in place, else from a new
 * group of the expected size (first_group_blocks, default 64, shrunk to the free run that is
 * there; plus reserve_tail blocks of headroom), else - when no free group is left - from the
 * tail of a randomly chosen other request's active group (seeded splitmix64), all of it or
 * max(need, half).  Ids are written to out_blocks[n_blocks] in logical order.  KV_ENOMEM_GPU
 * (nothing changes) if free blocks and other requests' tails together are fewer than n_blocks.
 * kv_bg_table returns the current table (ids of the used blocks in logical order; *out_n is the
 * length even when cap is smaller).  kv_bg_close returns every block of the request, tails
 * included; blocks an unfinished gather still reads stay unavailable until it has finished.
 * Shares the free lists with alloc_block_group / free_block_group. */
typedef struct {
  int64_t n_requests, n_groups /* with at least one used block */, used_blocks, tail_blocks;
  int64_t steals, opened, appended_groups, grown_in_place;
} kv_bg_stats_t;
int32_t kv_bg_configure(kv_pool_t* pool, int32_t first_group_blocks /* 0 = 64 */, uint64_t seed);
int32_t kv_bg_append(kv_pool_t* pool, int64_t req, int32_t n_blocks, int32_t reserve_tail,
                     int32_t* out_blocks);
int32_t kv_bg_table(kv_pool_t* pool, int64_t req, int32_t* out_blocks, int32_t cap, int32_t* out_n);
int32_t kv_bg_close(kv_pool_t* pool, int64_t req);
int32_t kv_bg_stats(kv_pool_t* pool, kv_bg_stats_t* out);

/* Sections 2.1 / 3.3.  Full swap-out: every logical block j (block_table[j] = its physical
 * id) is copied into the request's host image, replacing any earlier image.
 * KV_EINVAL: id out of range or repeated.  KV_ENOMEM_HOST: arena full. */
int32_t swap_out(kv_pool_t* pool, int64_t req, const int32_t* block_table, int32_t n_blocks);
/* Section 3.3.  Swap-out with reuse: moves exactly the logical blocks j with
 * dirty_mask[j] != 0 or without a valid host copy; all other image bytes stay.  A request
 * longer than its image has the image extended (in place when the reserved slack or the
 * neighbouring arena space allows, else by a further extent).  n_blocks smaller than the image
 * is KV_EINVAL.  out_n_moved may be NULL. */
int32_t swap_out_delta(kv_pool_t* pool, int64_t req, const int32_t* block_table, int32_t n_blocks,
                       const uint8_t* dirty_mask, int32_t* out_n_moved);
/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  A variant of swap_out that allocates nothing, on the device or
 * through any library, and keeps no state: the gather kernel packs the listed blocks into a
 * staging array that is part of the library's code object (KV_STATIC_STAGING_BYTES = 64 MiB,
 * held by every GPU the library runs on until the process ends; its address on the pool's
 * device is looked up once, in kv_pool_create), and one copy takes them from there to
 * host_dst, both enqueued on `stream`.  host_dst: caller-owned host memory, pinned for the
 * copy to be asynchronous, n_blocks * R bytes, layout dst[j][p][C] (the host-image layout).
 * stream: the caller's hipStream_t; NULL = a stream of the library, and the call then
 * returns when the bytes have arrived.  No request, no host image, no reuse map and no
 * conflict tracking are involved: ordering against other work on the blocks is the
 * caller's, by stream order.
 * Limits: n_blocks <= 896 and n_blocks * R <= 64 MiB, else KV_EINVAL (nothing is enqueued).
 * KV_EINVAL also for ids out of range or repeated; KV_ENODEV in a plan-only pool.
 * All calls on one GPU share the one staging array, which keeps the last call's bytes: calls
 * whose device work overlaps on one GPU (different streams, or several pools) race. */
int32_t swap_out_static(kv_pool_t* pool, const int32_t* block_table, int32_t n_blocks, void* host_dst,
                        void* stream);

/* Section 3.2 swap-in path.  Copies the host image into new_block_table's blocks.  The
 * image is kept (Section 3.3).  Note: any order of calls is correct, and when one scheduling step
 * both resumes and preempts, the resumed request is back equally soon whether its swap-in is issued
 * before or after the step's swap-out - except in a KV_FLAG_NO_DEFER_COPIES pool, where calls reach the
 * copy engines in call order and the swap-in should go first (Algorithm 1's order, which
 * kv_manager_iterate follows in any case).  A swap-in of a request whose swap-out has just been issued
 * first waits, on the host, until that swap-out's copies have been enqueued.
 * KV_ENOENT: no image, or a needed block's host copy is not valid.  KV_EINVAL: n_blocks differs from
 * the image, bad ids. */
int32_t swap_in(kv_pool_t* pool, int64_t req, const int32_t* new_block_table, int32_t n_blocks);
/* As swap_in, but logical blocks with resident_mask[j] != 0 are already on the GPU and are
 * skipped (only non-resident blocks move). */
int32_t swap_in_delta(kv_pool_t* pool, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                      const uint8_t* resident_mask, int32_t* out_n_moved);

/* Batched forms: one scheduling iteration preempts / resumes several requests (Algorithm 1,
 * steps 2 and 3).  tables is the concatenation of the requests' block tables,
 * n_blocks[i] the length of request i's.  All requests are validated first; pack kernels
 * and copies are shared across request boundaries.  A request id may appear once. */
int32_t swap_out_batch(kv_pool_t* pool, int32_t n_req, const int64_t* reqs,
                       const int32_t* tables, const int32_t* n_blocks);
int32_t swap_in_batch(kv_pool_t* pool, int32_t n_req, const int64_t* reqs,
                      const int32_t* tables, const int32_t* n_blocks);

/* Comparison path, measured for context only: the paper's own transfer scheme (Section 3.1:
 * one copy per contiguous block group; per_block != 0: one copy per block, the baseline of
 * Section 2.2) applied to this pool layout, with no pack kernel - one 2-D copy per (run of
 * physically adjacent blocks, plane) straight between the pool and the host image.  Same
 * result, same validation and reuse-map effects as swap_out / swap_in. */
int32_t swap_out_direct(kv_pool_t* pool, int64_t req, const int32_t* block_table, int32_t n_blocks,
                        int32_t per_block);
int32_t swap_in_direct(kv_pool_t* pool, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                       int32_t per_block);

/* Layer-wise swap-in: the alternative Section 2.2 (Challenge #2) discusses, layer-wise
 * asynchronous swapping as in earlier systems, built on this path for comparison.  Same result,
 * validation and reuse-map effects as swap_in_delta (resident_mask may be NULL: move
 * everything; out_n_moved may be NULL), but the KV arrives in steps of layers_per_step layers
 * (1 .. n_layers), lowest layers first: per step one 2-D host-to-device copy per run of
 * adjacent host records (the K and V planes of consecutive layers are one contiguous slice of
 * each record) and one scatter over that plane range; in a KV_FLAG_MAPPED_SWAP_IN pool a step
 * is instead one launch of the kernel that reads the pinned image directly, over that plane
 * range (no copies, no staging).  kv_stream_wait_layer makes a
 * hipStream_t wait on the device, kv_wait_layer the calling thread, until the step that holds
 * `layer` has landed, so attention over layer l can start while the layers above it are still
 * on the link.  For a request whose last op is not a layer-wise swap-in both wait for that
 * whole op.  KV_EINVAL for a layer outside [0, n_layers). */
int32_t swap_in_layerwise(kv_pool_t* pool, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                          const uint8_t* resident_mask, int32_t layers_per_step, int32_t* out_n_moved);
int32_t kv_stream_wait_layer(kv_pool_t* pool, int64_t req, int32_t layer, void* stream);
int32_t kv_wait_layer(kv_pool_t* pool, int64_t req, int32_t layer);

/* Completion (Algorithm 1, step 1: IsCompleted / Synchronize).  KV_ENOENT for a request the
 * library does not know: one never swapped, or whose host copy was released. */
int32_t kv_wait(kv_pool_t* pool, int64_t req);                /* blocks until req's last op is done */
int32_t kv_query(kv_pool_t* pool, int64_t req, int32_t* done);/* non-blocking; *done = 0/1 */
int32_t kv_wait_packed(kv_pool_t* pool, int64_t req);         /* until the last swap-out's gather has
                                                                 finished: GPU blocks reusable */
int32_t kv_stream_wait(kv_pool_t* pool, int64_t req, void* stream); /* make a hipStream_t wait (on the
                                                                 device) for req's last op */
int32_t kv_wait_all(kv_pool_t* pool);  /* until everything enqueued before the call is done; other
                                          threads may keep calling meanwhile */

/* Reuse map (Section 3.3). */
/* The image of a request is a list of extents of the pinned arena: one extent (with slack
 * behind it) when it is created, a further extent whenever it grows past the room reserved
 * and the arena space behind it is taken - an image is never moved.  kv_host_len reports
 * its length and extent count; kv_host_blocks reports where each logical block is:
 * record_index[j] (caller-allocated, n = image length) is the index of the R-byte record
 * [P][C] of logical block j, i.e. its bytes start at *arena_base + record_index[j]*R
 * (-1: the block has no record because its space was reclaimed; its host_valid bit is 0).
 * Consecutive logical blocks are adjacent inside an extent.  Valid until the image is
 * released or rebuilt by a full swap_out; wait for the request before reading the bytes.
 * In a KV_FLAG_PLAN_ONLY pool *arena_base is NULL (there are no bytes), the indices are real. */
int32_t kv_host_len(kv_pool_t* pool, int64_t req, int32_t* n_blocks, int32_t* n_extents);
int32_t kv_host_blocks(kv_pool_t* pool, int64_t req, const void** arena_base, int64_t* record_index,
                       int32_t n);
/* Section 3.3: the CPU copy itself, in the layout of the contract.  kv_host_read copies logical
 * blocks [first_block, first_block + n_blocks) of req's image into dst (host memory,
 * n_blocks * R bytes, caller-owned) as dst[j - first_block][p][C], whatever extents the
 * records sit in; a block whose record was reclaimed reads as zeros (its host_valid bit is 0).
 * It waits for the request's last op first, and holds the pool's lock while it copies (a
 * reading aid for tests, tools and checkpointing, not a hot-path call).  KV_ENODEV in a
 * plan-only pool.
 * kv_host_view is the zero-copy form: *bytes = n * R, and *ptr = the image's first byte when
 * all its records are consecutive in the arena (one extent, nothing reclaimed), NULL
 * otherwise (then use kv_host_read).  Valid until the image grows, is released or rebuilt;
 * it does not wait - use kv_wait before reading through it. */
int32_t kv_host_read(kv_pool_t* pool, int64_t req, int32_t first_block, int32_t n_blocks, void* dst);
int32_t kv_host_view(kv_pool_t* pool, int64_t req, const void** ptr, int64_t* bytes);
int32_t kv_host_valid(kv_pool_t* pool, int64_t req, uint8_t* out_mask, int32_t n); /* 1 = valid */
int32_t kv_host_invalidate(kv_pool_t* pool, int64_t req, const uint8_t* mask, int32_t n); /* contaminate */
int32_t kv_host_release(kv_pool_t* pool, int64_t req);        /* drop the image (waits for its ops) */
int32_t kv_host_set_priority(kv_pool_t* pool, int64_t req, int32_t priority); /* default 0; used by
                                                                 KV_FLAG_HOST_EVICT */

typedef struct {
  int64_t bytes_out, bytes_in;          /* payload bytes enqueued per direction (moved blocks * R) */
  int64_t blocks_out, blocks_in;
  int64_t gather_launches, scatter_launches;
  int64_t d2h_copies, h2d_copies;
  int64_t conflict_waits;               /* device-side waits inserted by conflict detection */
  int64_t host_new_extents;             /* image growths that had to open a new arena extent */
  int64_t host_evicted_blocks;          /* logical blocks whose host copy was reclaimed (KV_FLAG_HOST_EVICT) */
  int64_t host_arena_used, host_arena_bytes;
  int64_t strided_copies;               /* of d2h_copies + h2d_copies: 2-D copies that carry several runs */
  int64_t second_lane_copies;           /* of d2h_copies: issued on the host-to-device stream (KV_FLAG_SECOND_LANE) */
} kv_stats_t;
int32_t kv_stats(kv_pool_t* pool, kv_stats_t* out);

/* Profiling (needs KV_FLAG_PROFILE).  One record per kernel launch / copy, in issue order. */
typedef struct {
  int32_t kind;      /* 0 gather, 1 scatter, 2 D2H copy, 3 H2D copy, 4 mapped swap-in kernel, 5 mapped swap-out kernel */
  int32_t reserved;
  int64_t bytes;     /* payload bytes of this launch / copy */
  double  ms;        /* device duration */
  double  start_ms;  /* when it began, relative to the first record's beginning */
} kv_prof_record_t;
/* Waits for all work, then writes up to cap records; *out_n = number available. */
int32_t kv_profile_read(kv_pool_t* pool, kv_prof_record_t* out, int32_t cap, int32_t* out_n);
int32_t kv_profile_reset(kv_pool_t* pool);

/* Host-link probe: times `reps` pinned copies of `bytes` bytes on a side stream and
 * returns the best rate in GB/s.  direction 0 = device-to-host, 1 = host-to-device,
 * 2 = both at once (sum).  Defines the "measured host-link peak". */
int32_t kv_link_probe(int64_t bytes, int32_t direction, int32_t reps, double* out_gbps);
/* Device copy ceiling: plain device-to-device copy kernel, read+write GB/s. */
int32_t kv_hbm_probe(int64_t bytes, int32_t reps, double* out_gbps);

/* R = bytes of one block record (all planes of one block). */
int32_t kv_record_bytes(kv_pool_t* pool, int64_t* out);

/* ---------------------------------------------------------------------------------------
 * Swap manager (Section 3.2, Algorithm 1): dispatch of swaps on a thread of its own.
 * submit copies the table and returns at once; a dispatcher thread calls the pool's entry
 * points in submission order (the order conflict detection relies on); poll reports tasks
 * whose device work has finished (Algorithm 1, step 1); wait / drain are the Synchronize
 * steps; strategy is step 4's choice between asynchronous and synchronous swap-in.
 * One dispatcher is enough here: a swap is a handful of runtime calls, not one per block
 * group.  The manager does not own the pool; destroy the manager first. */
typedef struct kv_manager kv_manager_t;

#define KV_TASK_SWAP_OUT       0
#define KV_TASK_SWAP_IN        1
#define KV_TASK_SWAP_OUT_DELTA 2 /* mask = dirty mask */
#define KV_TASK_SWAP_IN_DELTA  3 /* mask = resident mask */

typedef struct {
  int32_t window;        /* r_info: how many recent swaps the strategy remembers; <= 0: 64 */
  int32_t reserved;
  double  link_gbps;     /* host-link rate the strategy uses to estimate swap-in time; <= 0: 55 */
  double  sync_below_ms; /* swap-ins estimated shorter than this are waited for (synchronous)
                            rather than tracked across iterations; <= 0: 0.5 */
} kv_manager_config_t;

typedef struct {
  int64_t submitted, dispatched, failed, queued, in_flight;
  int64_t strategy_calls, strategy_async;
  double  dispatch_us_sum;    /* time the dispatcher spent inside the pool's entry points */
  double  queue_wait_us_sum;  /* submit -> start of dispatch */
} kv_manager_stats_t;

int32_t kv_manager_create(kv_pool_t* pool, const kv_manager_config_t* cfg /* may be NULL */,
                          kv_manager_t** out);
int32_t kv_manager_destroy(kv_manager_t* mgr);  /* dispatches what is queued, waits for it */
/* kind = KV_TASK_*; table / mask as for the entry point of that kind (copied before return).
 * *ticket (may be NULL) names the task in poll / wait.  Validation errors of the entry point
 * are reported as the task's status, not here. */
int32_t kv_manager_submit(kv_manager_t* mgr, int32_t kind, int64_t req, const int32_t* table,
                          int32_t n_blocks, const uint8_t* mask, uint64_t* ticket);
/* Up to cap finished tasks (device work done, or dispatch failed): tickets[i], status[i]
 * (status may be NULL).  Non-blocking.  Each task is reported once, by poll or by wait. */
int32_t kv_manager_poll(kv_manager_t* mgr, uint64_t* tickets, int32_t* status, int32_t cap,
                        int32_t* n_out);
/* Blocks until the task has been dispatched and its device work is done. */
int32_t kv_manager_wait(kv_manager_t* mgr, uint64_t ticket, int32_t* status /* may be NULL */);
int32_t kv_manager_drain(kv_manager_t* mgr);    /* everything submitted so far is done */
/* Step 4: the scheduler wants n_swap_in requests of swap_in_blocks blocks in total back now.
 * *async_out = 1: let them proceed asynchronously and poll; 0: wait for them (stall). */
int32_t kv_manager_strategy(kv_manager_t* mgr, int32_t n_swap_in, int64_t swap_in_blocks,
                            int32_t* async_out);
int32_t kv_manager_stats(kv_manager_t* mgr, kv_manager_stats_t* out);

/* Algorithm 1 (Section 3.2) as one call per scheduler iteration.  The manager keeps the
 * algorithm's queues: every request it has seen is `running` (on the GPU), `swapped` (host
 * copy only) or in `ongoing_swap_in`.  The scheduler passes what it decided for this iteration:
 * the requests to resume with their new block tables, and the requests to preempt with their
 * block tables (and dirty masks, for swap-out with reuse; NULL = full swap-outs).  The call
 *   1. polls the swap-ins started by earlier iterations: those that have finished move from
 *      ongoing_swap_in to running and are written to resumed[];
 *   2. dispatches the swap-ins, 3. dispatches the swap-outs (through the dispatcher thread),
 *      recording both in the window of recent swaps (r_info);
 *   3.1 detects KV cache conflicts - a physical block that a swap-out of this iteration reads
 *      and a swap-in of this iteration overwrites - on the tables, before anything is
 *      dispatched: conflicting swap-outs are dispatched ahead of the swap-ins, and the pool
 *      makes exactly the scatters concerned wait for their gathers on the device (fine-
 *      grained synchronisation; the host never stalls for it);
 *   4. asks the strategy: asynchronous - the new swap-ins join ongoing_swap_in and the
 *      scheduler goes on; synchronous - the call waits for them (SwapInStreamSynchronize) and
 *      they are in resumed[] already.  force_mode 1 / 2 overrides the strategy (always
 *      asynchronous / always synchronous), 0 leaves it to kv_manager_strategy.
 * A request is preempted from `running` only (one the manager has never seen counts as
 * running), and resumed from `swapped` only: KV_EBUSY / KV_ENOENT otherwise, nothing is
 * dispatched then.  A swap that fails when it is dispatched (arena full, bad table) is booked
 * by the next call: the request returns to the queue it came from and is listed by
 * kv_manager_failures.  *n_resumed is the number of resumed requests even when cap is smaller. */
typedef struct {
  int32_t n_swap_in, n_swap_out;
  const int64_t* in_reqs;       /* [n_swap_in] */
  const int32_t* in_tables;     /* concatenated new block tables */
  const int32_t* in_n_blocks;   /* [n_swap_in] */
  const int64_t* out_reqs;      /* [n_swap_out] */
  const int32_t* out_tables;    /* concatenated block tables */
  const int32_t* out_n_blocks;  /* [n_swap_out] */
  const uint8_t* out_dirty;     /* concatenated dirty masks, or NULL */
  int32_t force_mode;           /* 0 strategy decides, 1 asynchronous, 2 synchronous */
  int32_t flags;                /* KV_IT_* */
} kv_iteration_t;
#define KV_IT_FREE_OUT_BLOCKS 1 /* preemption gives the victims' GPU blocks up: the dispatcher calls
                                   free_block_group(req, table) right after each swap-out is enqueued - the
                                   earliest moment at which the allocator knows to hold them back until the
                                   gather has read them.  (A scheduler that frees them itself must not do so
                                   before the swap-out has been dispatched.) */
typedef struct {
  int32_t completed_swap_ins;   /* step 1: ongoing swap-ins that had finished */
  int32_t waited_swap_ins;      /* step 4: swap-ins of this iteration the call waited for */
  int32_t async;                /* step 4 decision: 1 asynchronous, 0 synchronous */
  int32_t conflicts;            /* step 3.1: swap-outs of this iteration dispatched ahead of the swap-ins */
  int32_t ongoing_swap_ins;     /* length of ongoing_swap_in after the call */
  int32_t failures;             /* failed swaps waiting in kv_manager_failures */
} kv_iteration_result_t;
typedef struct {
  int64_t iterations, swap_ins, swap_outs, async_iterations, sync_iterations, conflicts, resumed;
} kv_iteration_stats_t;
#define KV_WHERE_RUNNING 0
#define KV_WHERE_SWAPPED 1
#define KV_WHERE_ONGOING_SWAP_IN 2
int32_t kv_manager_iterate(kv_manager_t* mgr, const kv_iteration_t* it, int64_t* resumed, int32_t cap,
                           int32_t* n_resumed, kv_iteration_result_t* result /* may be NULL */);
int32_t kv_manager_failures(kv_manager_t* mgr, int64_t* reqs, int32_t* status, int32_t cap, int32_t* n_out);
int32_t kv_manager_where(kv_manager_t* mgr, int64_t req, int32_t* where); /* KV_WHERE_*; KV_ENOENT: never seen */
int32_t kv_manager_iteration_stats(kv_manager_t* mgr, kv_iteration_stats_t* out);

/* Thread-local text of the last error. */
const char* kv_last_error(void);
const char* kv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVSWAP_H */
