// Device-side interface of the pack kernels (gfx950).  Internal to the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// A launch carries its slice of the block table inside the kernel arguments
// (HIP allows 4 KiB of them), so no table upload is ever enqueued.
#define KV_MAX_LAUNCH_BLOCKS 896
#define KV_WG 256  // lanes per workgroup of the linear copy probe

struct KvPackArgs {
  char* pool;            // device: pool[p][b][C]
  char* staging;         // device: staging[k][p][C], k = position in this launch's table
  int64_t plane_stride;  // N * C bytes
  uint32_t C;            // chunk bytes (multiple of 16)
  uint32_t P;            // planes
  uint32_t m;            // blocks in this launch (<= KV_MAX_LAUNCH_BLOCKS)
  uint32_t tiles_per_chunk;
  uint32_t n_tiles;      // m * P * tiles_per_chunk
  uint32_t xcd_blocks;   // XCD-aware order: blocks one XCD works on at a time (set by the launcher)
  int32_t table[KV_MAX_LAUNCH_BLOCKS];  // physical block id of each of the m blocks
};

// Swap-in straight from the pinned host image (no staging, no copy engine): the launch's
// table pairs each block's physical id with the arena record that holds its bytes.
#define KV_MAX_MAPPED_BLOCKS 440
struct KvMappedArgs {
  char* pool;            // device: pool[p][b][C]
  char* host;            // device-visible address of the pinned arena
  int64_t plane_stride;  // N * C bytes
  int64_t R;             // record bytes = P * C
  uint32_t C;
  uint32_t P;
  uint32_t m;            // blocks in this launch (<= KV_MAX_MAPPED_BLOCKS)
  uint32_t tiles_per_chunk;
  uint32_t n_tiles;
  uint32_t pad;
  int32_t phys[KV_MAX_MAPPED_BLOCKS];
  uint32_t rec[KV_MAX_MAPPED_BLOCKS];
};
// grid: workgroups (few: the host link, not the CUs, is the limit).
// to_host: records go from the pool to the arena (swap-out); else from the arena to the pool.
hipError_t kv_launch_mapped(bool to_host, const KvMappedArgs& a, int grid, hipStream_t stream,
                            hipEvent_t start, hipEvent_t stop);

#define KV_PACK_TILE 0        // one tile per workgroup, 256 lanes; XCD-aware order for launches of
                              // KV_XCD_MIN_BLOCKS blocks or more, 3-D grid below (default)
#define KV_PACK_PERSISTENT 1  // grid-stride loop, block table staged in LDS, 256 lanes
#define KV_PACK_TILE_256 2    // tile kernel, 256 lanes, always the plain 3-D grid
#define KV_XCD_MIN_BLOCKS 64  // smaller launches would leave XCDs without work in that order
#define KV_PACK_TILE_1024 3   // tile kernel, 1024 lanes

// unroll: 16-byte vectors per lane per tile (1, 2, 4 or 8); 0 picks from the chunk size.
// variant: KV_PACK_*.  grid: workgroups of the persistent variant (<= 0: 2048).
// start/stop may be null; when given they receive the dispatch's own begin / end timestamps.
hipError_t kv_launch_pack(bool scatter, const KvPackArgs& a, int unroll, int variant, int grid,
                          hipStream_t stream, hipEvent_t start, hipEvent_t stop);
// Most blocks one launch may carry for this shape (table capacity and dispatch size).
int64_t kv_max_launch_blocks(uint32_t C, uint32_t P, int unroll, int variant);
// Plain linear device copy (bandwidth probe): bytes must be a multiple of 16.
hipError_t kv_launch_linear_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream,
                                 hipEvent_t start, hipEvent_t stop);
int kv_pick_unroll(uint32_t C, int wg);

// Staging for callers that may not allocate: a file-scope device array that every GPU the
// library runs on holds until the process ends.  kv_static_staging() returns its address on
// the CURRENT device (looked up once per device; null + an error code if that fails).
#define KV_STATIC_STAGING_BYTES (64ll << 20)
hipError_t kv_static_staging(char** ptr);
