// Gather / scatter pack kernels for paged KV blocks on gfx950 (CDNA4).
//
// A swap moves whole blocks of a request's KV cache (FastSwitch, arXiv 2411.18424,
// Section 2.2 Challenge #1: the block is the unit of allocation and transfer).  The pool
// keeps each (plane, block) chunk of C bytes contiguous, so a block is P chunks C bytes
// apart by a plane stride.  The gather kernel copies the P chunks of each listed block
// into one contiguous record of the staging buffer; the scatter kernel is its inverse.
// Pure data movement: no arithmetic on the payload, 64-bit addressing, 16 bytes per lane,
// non-temporal loads and stores (nothing is reused).
//
// Two decompositions are kept, selected per launch:
//
//  TILE (default): one workgroup of WG lanes moves one tile of WG*16*U contiguous bytes of one
//    chunk and exits.  The grid is 3-D, x = tile in chunk, y = plane, z = block of this launch, so
//    no index arithmetic is needed, consecutive workgroups walk the staging side linearly,
//    and the physical block id is one scalar load from the kernel arguments.  Letting the
//    hardware dispatcher do the looping measured ~12 % faster on MI355X than a persistent
//    grid-stride loop (about 6.2 vs 5.5 TB/s read+write on 1.75 GiB launches).
//
//  TILE, XCD-aware order (default for launches of 64 blocks or more): the same tiles through a
//    1-D grid.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so
//    workgroup w runs on XCD w % 8 (confirmed by reading XCC_ID in a probe kernel); the mapping gives every XCD two blocks of the launch at a
//    time (one where a block record is 4 MiB or more, see kv_xcd_blocks) and lets it walk them
//    chunk by chunk, alternating between the two (plane 0 of block A, plane 0 of block B, plane 1
//    of A ...), instead of spreading every chunk's tiles over all XCDs.  Measured on MI355X on the Llama-3-8B shape (896-block launches, read+write):
//    gather 6.57 against 6.18 TB/s, scatter 6.52 against 5.99 TB/s with block groups of 8, and
//    6.34 against 5.91 / 6.04 against 5.82 with fully fragmented tables; one block per XCD gives
//    6.37 / 6.32, four 6.38 / 6.41, eight 6.18 / 6.13, whole chunks per XCD 5.70 / 5.95.
//
//  PERSISTENT: a fixed grid of workgroups walks the tiles grid-strided; the launch's block
//    table slice is staged in LDS once per workgroup and each tile costs one LDS read.
//    Kept for comparison and for launches whose grid would not fit a 3-D dispatch.

#include "kv_kernels.h"

#include <hip/hip_ext.h>

#include <algorithm>
#include <mutex>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Streaming store of one vector to device memory: non-temporal and at agent scope (sc1).
// Measured on MI355X (read+write TB/s, 4 KiB per workgroup, nt loads; all 8 x 8 combinations of
// sc0 / sc1 / nt on loads and stores were swept): a plain 2 GiB copy reaches 6.65 with sc1
// stores against 6.43 with nt-only stores, the scatter (linear reads, writes strided over
// planes) 6.03 against 5.74; the gather (strided reads, linear writes) loses in plain 3-D order
// (5.74 against 6.19) and gains in XCD-aware order (6.80 against 6.69).  See store_policy().
// Loads: nt is what matters (6.1 without), the scope bits make no difference.
__device__ __forceinline__ void store_stream(u32x4 v, u32x4* p) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}

template <bool SC1>
__device__ __forceinline__ void store_vec(u32x4 v, u32x4* p) {
  if (SC1)
    store_stream(v, p);
  else
    __builtin_nontemporal_store(v, p);
}

template <int WG, int U, bool FULL, bool SCATTER, bool SC1>
__device__ __forceinline__ void move_tile(u32x4* pool_ptr, u32x4* stag_ptr, uint32_t rem) {
  const u32x4* src = SCATTER ? stag_ptr : pool_ptr;
  u32x4* dst = SCATTER ? pool_ptr : stag_ptr;
  u32x4 r[U];
  if (FULL) {
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(src + threadIdx.x + u * WG);
#pragma unroll
    for (int u = 0; u < U; ++u) store_vec<SC1>(r[u], dst + threadIdx.x + u * WG);
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * WG;
      if (i < rem) r[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * WG;
      if (i < rem) store_vec<SC1>(r[u], dst + i);
    }
  }
}

template <int WG, int U, bool FULL, bool SCATTER, bool SC1>
__global__ __launch_bounds__(WG) void kv_pack_tile_kernel(const KvPackArgs a) {
  constexpr uint32_t TILE_VECS = WG * U;  // 16-byte vectors per tile
  const uint32_t t = blockIdx.x, p = blockIdx.y, k = blockIdx.z;
  const int64_t b = a.table[k];  // wave-uniform: a scalar load from the kernel arguments
  const uint32_t v0 = t * TILE_VECS;
  u32x4* pool_ptr =
      reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + b * (int64_t)a.C) + v0;
  u32x4* stag_ptr =
      reinterpret_cast<u32x4*>(a.staging + ((int64_t)k * a.P + p) * (int64_t)a.C) + v0;
  move_tile<WG, U, FULL, SCATTER, SC1>(pool_ptr, stag_ptr, (a.C >> 4) - v0);
}

// The tile kernel in XCD-aware order: grid = groups of 8 XCDs x (K blocks' tiles), K = a.xcd_blocks
// blocks per XCD at a time (see kv_xcd_blocks).
constexpr uint32_t KV_XCDS = 8;

template <int WG, int U, bool FULL, bool SCATTER, bool SC1>
__global__ __launch_bounds__(WG) void kv_pack_xcd_kernel(const KvPackArgs a) {
  constexpr uint32_t TILE_VECS = WG * U;
  const uint32_t w = blockIdx.x, xcd = w % KV_XCDS, slot = w / KV_XCDS;
  const uint32_t tpc = a.tiles_per_chunk, K = a.xcd_blocks;
  const uint32_t per = K * tpc * a.P;           // tiles of the blocks one XCD holds
  const uint32_t g = slot / per, r = slot - g * per;
  const uint32_t c = r / tpc, t = r - c * tpc;  // chunk among the XCD's blocks, tile in it
  const uint32_t k = (g * KV_XCDS + xcd) * K + c % K, p = c / K;
  if (k >= a.m) return;  // the last group may be short
  const int64_t b = a.table[k];
  const uint32_t v0 = t * TILE_VECS;
  u32x4* pool_ptr =
      reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + b * (int64_t)a.C) + v0;
  u32x4* stag_ptr =
      reinterpret_cast<u32x4*>(a.staging + ((int64_t)k * a.P + p) * (int64_t)a.C) + v0;
  move_tile<WG, U, FULL, SCATTER, SC1>(pool_ptr, stag_ptr, (a.C >> 4) - v0);
}

template <int WG, int U, bool FULL, bool SCATTER, bool SC1>
__global__ __launch_bounds__(WG) void kv_pack_persistent_kernel(const KvPackArgs a) {
  __shared__ int32_t s_table[KV_MAX_LAUNCH_BLOCKS];
  for (uint32_t i = threadIdx.x; i < a.m; i += WG) s_table[i] = a.table[i];
  __syncthreads();

  constexpr uint32_t TILE_VECS = WG * U;
  const uint32_t tpc = a.tiles_per_chunk;
  const uint32_t P = a.P;
  for (uint32_t w = blockIdx.x; w < a.n_tiles; w += gridDim.x) {
    const uint32_t q = w / tpc;      // chunk number in staging order: q = k*P + p
    const uint32_t t = w - q * tpc;  // tile inside the chunk
    const uint32_t k = q / P;
    const uint32_t p = q - k * P;
    const int64_t b = s_table[k];
    const uint32_t v0 = t * TILE_VECS;
    u32x4* pool_ptr =
        reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + b * (int64_t)a.C) + v0;
    u32x4* stag_ptr = reinterpret_cast<u32x4*>(a.staging + (int64_t)q * a.C) + v0;
    move_tile<WG, U, FULL, SCATTER, SC1>(pool_ptr, stag_ptr, (a.C >> 4) - v0);
  }
}

// Swap without staging: a small persistent grid moves block records straight between the
// pool and pinned host memory; the table (physical id, arena record) of the launch is staged
// in LDS once per workgroup, 8 vectors per lane are in flight.
// TO_HOST = false (swap-in): loads travel over the host link, stores go to the pool.  A few
//   dozen workgroups saturate the link and host reads cost an HBM-bound neighbour only ~2 %.
// TO_HOST = true (swap-out): loads from the pool, stores to host memory.  Lowest latency for
//   small requests (one launch, no copy), but stores to the host back up the memory fabric:
//   an HBM-bound kernel beside it loses most of its bandwidth, so large transfers belong on
//   the copy engines.
template <bool FULL, bool TO_HOST>
__global__ __launch_bounds__(256) void kv_mapped_kernel(const KvMappedArgs a) {
  __shared__ int32_t s_phys[KV_MAX_MAPPED_BLOCKS];
  __shared__ uint32_t s_rec[KV_MAX_MAPPED_BLOCKS];
  for (uint32_t i = threadIdx.x; i < a.m; i += 256) {
    s_phys[i] = a.phys[i];
    s_rec[i] = a.rec[i];
  }
  __syncthreads();
  constexpr int U = 8;
  constexpr uint32_t TILE_VECS = 256 * U;
  const uint32_t tpc = a.tiles_per_chunk;
  const uint32_t P = a.P;
  const uint32_t chunk_vecs = a.C >> 4;
  for (uint32_t w = blockIdx.x; w < a.n_tiles; w += gridDim.x) {
    const uint32_t q = w / tpc;  // q = k*P + p: tiles walk each host record front to back
    const uint32_t t = w - q * tpc;
    const uint32_t k = q / P;
    const uint32_t p = q - k * P;
    const uint32_t v0 = t * TILE_VECS;
    u32x4* host = reinterpret_cast<u32x4*>(a.host + (int64_t)s_rec[k] * a.R + (int64_t)p * a.C) + v0;
    u32x4* pool = reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + (int64_t)s_phys[k] * a.C) + v0;
    const uint32_t rem = chunk_vecs - v0;
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * 256;
      if (FULL || i < rem) r[u] = TO_HOST ? __builtin_nontemporal_load(pool + i) : host[i];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * 256;
      if (FULL || i < rem) {
        if (TO_HOST)
          host[i] = r[u];
        else
          store_stream(r[u], pool + i);
      }
    }
  }
}

// Plain linear copy, one 4 KiB tile per workgroup: the device-copy ceiling the pack
// kernels are compared with.
__global__ __launch_bounds__(KV_WG) void kv_linear_copy_kernel(u32x4* __restrict__ dst,
                                                               const u32x4* __restrict__ src,
                                                               int64_t n_vecs) {
  const int64_t i = (int64_t)blockIdx.x * KV_WG + threadIdx.x;
  if (i < n_vecs) store_stream(__builtin_nontemporal_load(src + i), dst + i);
}

// Workgroup size of the tile kernel: 256 lanes (4 KiB tiles).  Measured on MI355X: alone, the
// gather is fastest with 256 lanes and the scatter ~2 % faster with 1024 lanes (16 KiB tiles);
// but beside a GEMM that fills the CUs a 1024-lane workgroup needs 16 free wave slots at once
// and the scatter drops to half the rate of the 256-lane one (0.6 vs 1.2 TB/s), so 256 lanes
// are the default for both directions.  64-lane workgroups do better still beside a GEMM
// (gather 3.4 vs 2.2 TB/s) but lose 12 % alone.
// Store policy of a launch: 1 = sc1 nt, 0 = nt only.  The scatter always stores with sc1 nt;
// the gather does in XCD-aware order (+1.5 %) and does not in plain 3-D order (-5 %).  Variants
// 4 .. 7 force the four combinations (bit 0: gather stores sc1, bit 1: scatter stores sc1).
static int store_policy(int variant, bool scatter, bool xcd_order) {
  int bits = xcd_order ? 3 : 2;
  if (variant >= 4 && variant <= 7) bits = variant - 4;
  return scatter ? (bits >> 1) & 1 : bits & 1;
}

// Blocks one XCD works on at a time in XCD-aware order.  Measured on MI355X (read+write TB/s,
// gather / scatter): Llama-3-8B shape (record 2 MiB, 16 GiB pool) one block 6.75 / 6.49, two 6.84 /
// 6.59, four 6.68 / 6.42; Qwen2-72B shape (record 5 MiB, 236 GB pool) one 6.16 / 6.76 - 6.82, two
// 6.04 - 6.13 / 6.49 - 6.67, four 5.93 - 6.10 / 6.16 - 6.60; Llama-2-13B shape (record 12.5 MiB,
// 230 GB pool) one 6.27 / 6.67, two 6.18 / 6.38, four 6.13 / 6.13.  An XCD wants about 4 MiB of
// records in hand: two blocks while a record is smaller than that, one block otherwise.
static uint32_t kv_xcd_blocks(uint32_t C, uint32_t P) { return (uint64_t)C * P >= (4u << 20) ? 1u : 2u; }

static int pick_wg(int variant) { return variant == KV_PACK_TILE_1024 ? 1024 : 256; }

int kv_pick_unroll(uint32_t C, int wg) {
  // one vector per lane measured fastest
  if (C % (uint32_t)(wg * 16) == 0) return 1;
  return 0;  // the tile does not divide the chunk: the bounds-checked kernel is used
}

struct Shape {
  int wg, U;
  bool full;
  uint32_t tpc;
};

static Shape pick_shape(uint32_t C, int unroll, int variant, bool scatter) {
  Shape s;
  (void)scatter;
  s.wg = pick_wg(variant);
  s.U = unroll;
  if (s.U != 1 && s.U != 2 && s.U != 4 && s.U != 8) s.U = kv_pick_unroll(C, s.wg);
  if (s.wg == 1024 && s.U > 2) s.U = 2;  // 1024-lane tiles exist for one and two vectors per lane
  s.full = s.U != 0 && C % (uint32_t)(s.wg * 16 * s.U) == 0;
  if (s.U == 0) s.U = 1;
  const uint32_t tile = (uint32_t)s.wg * 16u * (uint32_t)s.U;
  s.tpc = (C + tile - 1) / tile;
  return s;
}

int64_t kv_max_launch_blocks(uint32_t C, uint32_t P, int unroll, int variant) {
  // keep both directions' dispatches below 2^31 work-items
  const Shape g = pick_shape(C, unroll, variant, false), sc = pick_shape(C, unroll, variant, true);
  const uint64_t items = std::max<uint64_t>((uint64_t)g.wg * g.tpc, (uint64_t)sc.wg * sc.tpc);
  uint64_t by_grid = (1ull << 31) / (items * P);
  if (by_grid < 1) by_grid = 1;
  return (int64_t)(by_grid < KV_MAX_LAUNCH_BLOCKS ? by_grid : KV_MAX_LAUNCH_BLOCKS);
}

enum LaunchMode { MODE_TILE_3D = 0, MODE_PERSISTENT = 1, MODE_TILE_XCD = 2 };

// The extended launch attaches the dispatch's own begin / end timestamps to two events; without
// events the plain launch is used (which a stream capture records like any other kernel node).
#define KV_LAUNCH(kernel, grid_dim, block_dim)                                                    \
  do {                                                                                            \
    if (start || stop)                                                                            \
      hipExtLaunchKernelGGL(kernel, grid_dim, block_dim, 0, stream, start, stop, 0, a);           \
    else                                                                                          \
      hipLaunchKernelGGL(kernel, grid_dim, block_dim, 0, stream, a);                              \
  } while (0)

template <int WG, int U, bool FULL, bool SCATTER, bool SC1>
static hipError_t launch_one(const KvPackArgs& a, int mode, int grid, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop) {
  if (mode == MODE_PERSISTENT) {
    KV_LAUNCH((kv_pack_persistent_kernel<WG, U, FULL, SCATTER, SC1>), dim3(grid), dim3(WG));
  } else if (mode == MODE_TILE_XCD) {
    KV_LAUNCH((kv_pack_xcd_kernel<WG, U, FULL, SCATTER, SC1>), dim3(grid), dim3(WG));
  } else {
    KV_LAUNCH((kv_pack_tile_kernel<WG, U, FULL, SCATTER, SC1>), dim3(a.tiles_per_chunk, a.P, a.m), dim3(WG));
  }
  return hipGetLastError();
}

template <int WG, int U, bool SC1>
static hipError_t launch_wu(bool scatter, bool full, const KvPackArgs& a, int mode, int grid,
                            hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  if (scatter)
    return full ? launch_one<WG, U, true, true, SC1>(a, mode, grid, stream, start, stop)
                : launch_one<WG, U, false, true, SC1>(a, mode, grid, stream, start, stop);
  return full ? launch_one<WG, U, true, false, SC1>(a, mode, grid, stream, start, stop)
              : launch_one<WG, U, false, false, SC1>(a, mode, grid, stream, start, stop);
}

hipError_t kv_launch_pack(bool scatter, const KvPackArgs& a_in, int unroll, int variant, int grid,
                          hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  if (a_in.m == 0) return hipSuccess;
  if (a_in.m > KV_MAX_LAUNCH_BLOCKS || (a_in.C & 15u) || a_in.C == 0 || a_in.P == 0)
    return hipErrorInvalidValue;
  KvPackArgs a = a_in;
  const Shape s = pick_shape(a.C, unroll, variant, scatter);
  a.tiles_per_chunk = s.tpc;
  const uint64_t n_tiles = (uint64_t)a.m * a.P * a.tiles_per_chunk;
  if (n_tiles > 0xFFFFFFFFull) return hipErrorInvalidValue;
  a.n_tiles = (uint32_t)n_tiles;
  int mode = variant == KV_PACK_PERSISTENT ? MODE_PERSISTENT : MODE_TILE_3D;
  // the 3-D grid needs y, z < 65536 and a dispatch below 2^31 work-items
  if (a.P > 65535u || n_tiles * (uint64_t)s.wg > (1ull << 31)) mode = MODE_PERSISTENT;
  if (grid <= 0) grid = 2048;
  if ((uint64_t)grid > n_tiles) grid = (int)n_tiles;
  if (mode == MODE_TILE_3D && variant != KV_PACK_TILE_256 && a.m >= KV_XCD_MIN_BLOCKS) {
    // XCD-aware order; the grid is padded to whole groups of 8 or 16 blocks
    a.xcd_blocks = kv_xcd_blocks(a.C, a.P);
    const uint64_t group = (uint64_t)KV_XCDS * a.xcd_blocks;
    const uint64_t padded = (a.m + group - 1) / group * group * a.P * a.tiles_per_chunk;
    if (padded * (uint64_t)s.wg <= (1ull << 31)) {
      mode = MODE_TILE_XCD;
      grid = (int)padded;
    }
  }
  const int policy = store_policy(variant, scatter, mode == MODE_TILE_XCD);
#define KV_CASE(WW, UU)                                                                             \
  if (s.wg == WW && s.U == UU)                                                                      \
    return policy ? launch_wu<WW, UU, true>(scatter, s.full, a, mode, grid, stream, start, stop) \
                  : launch_wu<WW, UU, false>(scatter, s.full, a, mode, grid, stream, start, stop);
  KV_CASE(256, 1)
  KV_CASE(256, 2)
  KV_CASE(256, 4)
  KV_CASE(256, 8)
  KV_CASE(1024, 1)
  KV_CASE(1024, 2)
#undef KV_CASE
  return hipErrorInvalidValue;
}

// Staging of the entry point that allocates nothing.  In host code this name is only a handle
// for hipGetSymbolAddress; kernels and copies get the address that call returns.
static __device__ __align__(256) unsigned char scratch[KV_STATIC_STAGING_BYTES];

hipError_t kv_static_staging(char** ptr) {
  constexpr int MAX_DEV = 64;
  static char* addr[MAX_DEV];  // per device: each GPU holds its own copy of the array
  static std::mutex mu;
  *ptr = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> g(mu);
  if (!addr[dev]) {
    void* a = nullptr;
    e = hipGetSymbolAddress(&a, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    addr[dev] = (char*)a;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

hipError_t kv_launch_linear_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream,
                                 hipEvent_t start, hipEvent_t stop) {
  if (bytes <= 0 || (bytes & 15)) return hipErrorInvalidValue;
  const int64_t n_vecs = bytes >> 4;
  const int64_t grid = (n_vecs + KV_WG - 1) / KV_WG;
  if (grid > 0x7FFFFFFFll / KV_WG * 2) return hipErrorInvalidValue;
  hipExtLaunchKernelGGL(kv_linear_copy_kernel, dim3((unsigned)grid), dim3(KV_WG), 0, stream, start,
                        stop, 0, reinterpret_cast<u32x4*>(dst), reinterpret_cast<const u32x4*>(src),
                        n_vecs);
  return hipGetLastError();
}

hipError_t kv_launch_mapped(bool to_host, const KvMappedArgs& a_in, int grid, hipStream_t stream,
                            hipEvent_t start, hipEvent_t stop) {
  if (a_in.m == 0) return hipSuccess;
  if (a_in.m > KV_MAX_MAPPED_BLOCKS || (a_in.C & 15u) || a_in.C == 0 || a_in.P == 0)
    return hipErrorInvalidValue;
  KvMappedArgs a = a_in;
  const uint32_t tile = 256u * 16u * 8u;
  a.tiles_per_chunk = (a.C + tile - 1) / tile;
  const uint64_t n_tiles = (uint64_t)a.m * a.P * a.tiles_per_chunk;
  if (n_tiles > 0xFFFFFFFFull) return hipErrorInvalidValue;
  a.n_tiles = (uint32_t)n_tiles;
  if (grid <= 0) grid = 64;
  if ((uint64_t)grid > n_tiles) grid = (int)n_tiles;
  const bool full = a.C % tile == 0;
#define KV_LAUNCH_MAPPED(FULL, TO_HOST)                                                              \
  hipExtLaunchKernelGGL((kv_mapped_kernel<FULL, TO_HOST>), dim3(grid), dim3(256), 0, stream, start, \
                        stop, 0, a)
  if (to_host) {
    if (full) KV_LAUNCH_MAPPED(true, true); else KV_LAUNCH_MAPPED(false, true);
  } else {
    if (full) KV_LAUNCH_MAPPED(true, false); else KV_LAUNCH_MAPPED(false, false);
  }
#undef KV_LAUNCH_MAPPED
  return hipGetLastError();
}
