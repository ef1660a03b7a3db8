// Gather / scatter pack kernels for paged KV blocks on gfx950 (CDNA4).
//
// A swap moves whole blocks of a request's KV cache (FastSwitch, arXiv 2411.18424,
// Section 2.2 Challenge #1: the block is the unit of allocation and transfer).  The pool
// keeps each (plane, block) chunk of C bytes contiguous, so a block is P chunks C bytes
// apart by a plane stride.  The gather kernel copies the P chunks of each listed block
// into one contiguous record of the staging buffer; the scatter kernel is its inverse.
// Pure data movement: no arithmetic on the payload, 64-bit addressing, 16 bytes per lane.
//
// Work decomposition: a tile is KV_WG*16*U contiguous bytes of one chunk.  Tiles are
// numbered so that the staging side is one linear stream (tile w sits at byte w*tile in
// staging when the tile divides the chunk); workgroups walk tiles grid-strided, so at any
// moment the live workgroups cover a contiguous window of staging and P windows of the
// pool.  The launch's block-table slice arrives in the kernel arguments and is staged in
// LDS once per workgroup; each tile then needs one LDS read for its physical block id.

#include "kv_kernels.h"
#include <hip/hip_ext.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U, bool FULL, bool SCATTER>
__global__ __launch_bounds__(KV_WG) void kv_pack_kernel(const KvPackArgs a) {
  __shared__ int32_t s_table[KV_MAX_LAUNCH_BLOCKS];
  for (uint32_t i = threadIdx.x; i < a.m; i += KV_WG) s_table[i] = a.table[i];
  __syncthreads();

  constexpr uint32_t TILE_VECS = KV_WG * U;  // 16-byte vectors per tile
  const uint32_t chunk_vecs = a.C >> 4;
  const uint32_t tpc = a.tiles_per_chunk;
  const uint32_t P = a.P;

  for (uint32_t w = blockIdx.x; w < a.n_tiles; w += gridDim.x) {
    const uint32_t q = w / tpc;        // chunk number in staging order: q = k*P + p
    const uint32_t t = w - q * tpc;    // tile inside the chunk
    const uint32_t k = q / P;
    const uint32_t p = q - k * P;
    const int64_t b = s_table[k];
    const uint32_t v0 = t * TILE_VECS;
    u32x4* pool_ptr =
        reinterpret_cast<u32x4*>(a.pool + (int64_t)p * a.plane_stride + b * (int64_t)a.C) + v0;
    u32x4* stag_ptr = reinterpret_cast<u32x4*>(a.staging + (int64_t)q * a.C) + v0;
    const u32x4* src = SCATTER ? stag_ptr : pool_ptr;
    u32x4* dst = SCATTER ? pool_ptr : stag_ptr;

    u32x4 r[U];
    if (FULL) {
#pragma unroll
      for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(src + threadIdx.x + u * KV_WG);
#pragma unroll
      for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], dst + threadIdx.x + u * KV_WG);
    } else {
      const uint32_t rem = chunk_vecs - v0;  // vectors left in this chunk
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
}

template <int U>
__global__ __launch_bounds__(KV_WG) void kv_linear_copy_kernel(u32x4* __restrict__ dst,
                                                               const u32x4* __restrict__ src,
                                                               int64_t n_vecs) {
  constexpr int64_t TILE_VECS = KV_WG * U;
  const int64_t n_full = n_vecs / TILE_VECS;
  for (int64_t w = blockIdx.x; w < n_full; w += gridDim.x) {
    const u32x4* s = src + w * TILE_VECS + threadIdx.x;
    u32x4* d = dst + w * TILE_VECS + threadIdx.x;
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(s + u * KV_WG);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], d + u * KV_WG);
  }
  if (blockIdx.x == 0) {
    for (int64_t i = n_full * TILE_VECS + threadIdx.x; i < n_vecs; i += KV_WG) dst[i] = src[i];
  }
}

int kv_pick_unroll(uint32_t C) {
  for (int u = 8; u >= 1; u >>= 1)
    if (C % (uint32_t)(KV_WG * 16 * u) == 0) return u;
  return 0;  // no tile divides the chunk: the bounds-checked kernel is used
}

template <int U, bool FULL, bool SCATTER>
static hipError_t launch_one(const KvPackArgs& a, int grid, hipStream_t stream, hipEvent_t start,
                             hipEvent_t stop) {
  hipExtLaunchKernelGGL((kv_pack_kernel<U, FULL, SCATTER>), dim3(grid), dim3(KV_WG), 0, stream,
                        start, stop, 0, a);
  return hipGetLastError();
}

template <int U, bool FULL>
static hipError_t launch_dir(bool scatter, const KvPackArgs& a, int grid, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop) {
  return scatter ? launch_one<U, FULL, true>(a, grid, stream, start, stop)
                 : launch_one<U, FULL, false>(a, grid, stream, start, stop);
}

hipError_t kv_launch_pack(bool scatter, const KvPackArgs& a_in, int unroll, int grid,
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
    if (U == 0) U = 2;
  }
  const uint32_t tile = KV_WG * 16u * (uint32_t)U;
  a.tiles_per_chunk = (a.C + tile - 1) / tile;
  const uint64_t n_tiles = (uint64_t)a.m * a.P * a.tiles_per_chunk;
  if (n_tiles > 0xFFFFFFFFull) return hipErrorInvalidValue;
  a.n_tiles = (uint32_t)n_tiles;
  if (grid <= 0) grid = 2048;
  if ((uint64_t)grid > n_tiles) grid = (int)n_tiles;
#define KV_CASE(UU)                                                                  \
  case UU:                                                                           \
    return full ? launch_dir<UU, true>(scatter, a, grid, stream, start, stop)        \
                : launch_dir<UU, false>(scatter, a, grid, stream, start, stop);
  switch (U) {
    KV_CASE(1)
    KV_CASE(2)
    KV_CASE(4)
    KV_CASE(8)
  }
#undef KV_CASE
  return hipErrorInvalidValue;
}

hipError_t kv_launch_linear_copy(void* dst, const void* src, int64_t bytes, int grid,
                                 hipStream_t stream, hipEvent_t start, hipEvent_t stop) {
  if (bytes <= 0 || (bytes & 15)) return hipErrorInvalidValue;
  if (grid <= 0) grid = 2048;
  hipExtLaunchKernelGGL((kv_linear_copy_kernel<8>), dim3(grid), dim3(KV_WG), 0, stream, start, stop,
                        0, reinterpret_cast<u32x4*>(dst), reinterpret_cast<const u32x4*>(src),
                        bytes >> 4);
  return hipGetLastError();
}
