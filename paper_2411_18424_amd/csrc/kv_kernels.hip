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
//  TILE (default): one workgroup moves one tile of KV_WG*16*U contiguous bytes of one chunk
//    and exits.  The grid is 3-D, x = tile in chunk, y = plane, z = block of this launch, so
//    no index arithmetic is needed, consecutive workgroups walk the staging side linearly,
//    and the physical block id is one scalar load from the kernel arguments.  Letting the
//    hardware dispatcher do the looping measured ~12 % faster on MI355X than a persistent
//    grid-stride loop (about 6.2 vs 5.5 TB/s read+write on 1.75 GiB launches).
//
//  PERSISTENT: a fixed grid of workgroups walks the tiles grid-strided; the launch's block
//    table slice is staged in LDS once per workgroup and each tile costs one LDS read.
//    Kept for comparison and for launches whose grid would not fit a 3-D dispatch.

#include "kv_kernels.h"

#include <hip/hip_ext.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U, bool FULL, bool SCATTER>
__device__ __forceinline__ void move_tile(u32x4* pool_ptr, u32x4* stag_ptr, uint32_t rem) {
  const u32x4* src = SCATTER ? stag_ptr : pool_ptr;
  u32x4* dst = SCATTER ? pool_ptr : stag_ptr;
  u32x4 r[U];
  if (FULL) {
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(src + threadIdx.x + u * KV_WG);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], dst + threadIdx.x + u * KV_WG);
  } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * KV_WG;
      if (i < rem) r[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = threadIdx.x + u * KV_WG;
      if (i < rem) __builtin_nontemporal_store(r[u], dst + i);
    }
  }
}

template <int U, bool FULL, bool SCATTER>
__global__ __launch_bounds__(KV_WG) void kv_pack_tile_kernel(const KvPackArgs a) {
  constexpr uint32_t TILE_VECS = KV_WG * U;  // 16-byte vectors per tile
  const uint32_t t = blockIdx.x, p = blockIdx.y, k = blockIdx.z;
  const int64_t b = a.table[k];  // wave-uniform: a scalar load from the kernel arguments
  const uint32_t v0 = t * TILE_VECS;
  u32x4* pool_ptr =
      reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + b * (int64_t)a.C) + v0;
  u32x4* stag_ptr =
      reinterpret_cast<u32x4*>(a.staging + ((int64_t)k * a.P + p) * (int64_t)a.C) + v0;
  move_tile<U, FULL, SCATTER>(pool_ptr, stag_ptr, (a.C >> 4) - v0);
}

template <int U, bool FULL, bool SCATTER>
__global__ __launch_bounds__(KV_WG) void kv_pack_persistent_kernel(const KvPackArgs a) {
  __shared__ int32_t s_table[KV_MAX_LAUNCH_BLOCKS];
  for (uint32_t i = threadIdx.x; i < a.m; i += KV_WG) s_table[i] = a.table[i];
  __syncthreads();

  constexpr uint32_t TILE_VECS = KV_WG * U;
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
    move_tile<U, FULL, SCATTER>(pool_ptr, stag_ptr, (a.C >> 4) - v0);
  }
}

// Plain linear copy, one 4 KiB tile per workgroup: the device-copy ceiling the pack
// kernels are compared with.
__global__ __launch_bounds__(KV_WG) void kv_linear_copy_kernel(u32x4* __restrict__ dst,
                                                               const u32x4* __restrict__ src,
                                                               int64_t n_vecs) {
  const int64_t i = (int64_t)blockIdx.x * KV_WG + threadIdx.x;
  if (i < n_vecs) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

int kv_pick_unroll(uint32_t C) {
  // one vector per lane measured fastest; wider tiles only pay when they divide the chunk
  // and the chunk is large enough to keep the grid modest
  if (C % (uint32_t)(KV_WG * 16) == 0) return 1;
  return 0;  // no tile divides the chunk: the bounds-checked kernel is used
}

int64_t kv_max_launch_blocks(uint32_t C, uint32_t P, int unroll) {
  int U = (unroll == 1 || unroll == 2 || unroll == 4 || unroll == 8) ? unroll : kv_pick_unroll(C);
  if (U == 0) U = 1;
  const uint64_t tile = (uint64_t)KV_WG * 16u * (uint64_t)U;
  const uint64_t tpc = (C + tile - 1) / tile;
  // keep the dispatch below 2^31 work-items
  uint64_t by_grid = (1ull << 31) / ((uint64_t)KV_WG * tpc * P);
  if (by_grid < 1) by_grid = 1;
  return (int64_t)(by_grid < KV_MAX_LAUNCH_BLOCKS ? by_grid : KV_MAX_LAUNCH_BLOCKS);
}

template <int U, bool FULL, bool SCATTER>
static hipError_t launch_one(const KvPackArgs& a, bool persistent, int grid, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop) {
  if (persistent) {
    hipExtLaunchKernelGGL((kv_pack_persistent_kernel<U, FULL, SCATTER>), dim3(grid), dim3(KV_WG), 0,
                          stream, start, stop, 0, a);
  } else {
    hipExtLaunchKernelGGL((kv_pack_tile_kernel<U, FULL, SCATTER>), dim3(a.tiles_per_chunk, a.P, a.m),
                          dim3(KV_WG), 0, stream, start, stop, 0, a);
  }
  return hipGetLastError();
}

template <int U, bool FULL>
static hipError_t launch_dir(bool scatter, const KvPackArgs& a, bool persistent, int grid,
                             hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  return scatter ? launch_one<U, FULL, true>(a, persistent, grid, stream, start, stop)
                 : launch_one<U, FULL, false>(a, persistent, grid, stream, start, stop);
}

hipError_t kv_launch_pack(bool scatter, const KvPackArgs& a_in, int unroll, int variant, int grid,
                          hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  if (a_in.m == 0) return hipSuccess;
  if (a_in.m > KV_MAX_LAUNCH_BLOCKS || (a_in.C & 15u) || a_in.C == 0 || a_in.P == 0)
    return hipErrorInvalidValue;
  KvPackArgs a = a_in;
  int U = unroll;
  if (U != 1 && U != 2 && U != 4 && U != 8) U = kv_pick_unroll(a.C);
  bool full = true;
  if (U == 0 || a.C % (uint32_t)(KV_WG * 16 * U) != 0) {
    full = false;
    if (U == 0) U = 1;
  }
  const uint32_t tile = KV_WG * 16u * (uint32_t)U;
  a.tiles_per_chunk = (a.C + tile - 1) / tile;
  const uint64_t n_tiles = (uint64_t)a.m * a.P * a.tiles_per_chunk;
  if (n_tiles > 0xFFFFFFFFull) return hipErrorInvalidValue;
  a.n_tiles = (uint32_t)n_tiles;
  bool persistent = variant == KV_PACK_PERSISTENT;
  // the 3-D grid needs y, z < 65536 and a dispatch below 2^31 work-items
  if (a.P > 65535u || n_tiles * KV_WG > (1ull << 31)) persistent = true;
  if (grid <= 0) grid = 2048;
  if ((uint64_t)grid > n_tiles) grid = (int)n_tiles;
#define KV_CASE(UU)                                                                          \
  case UU:                                                                                   \
    return full ? launch_dir<UU, true>(scatter, a, persistent, grid, stream, start, stop)    \
                : launch_dir<UU, false>(scatter, a, persistent, grid, stream, start, stop);
  switch (U) {
    KV_CASE(1)
    KV_CASE(2)
    KV_CASE(4)
    KV_CASE(8)
  }
#undef KV_CASE
  return hipErrorInvalidValue;
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
