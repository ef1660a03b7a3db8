// A C caller reads host images in the contract layout [n][P][C] through kv_host_read and
// kv_host_view, with no help from the Python binding.  Needs a GPU.  The pool is filled with
// a byte pattern that is a function of (plane, physical block, offset), requests are swapped
// out through permuted tables, one image is grown until it continues in a second extent, and
// every byte read back must be the pattern of the block the table names.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/kvswap.h"

static int g_fail = 0;
#define EXPECT(c, ...)                                              \
  do {                                                              \
    if (!(c)) {                                                     \
      fprintf(stderr, "FAIL %s:%d: %s: ", __FILE__, __LINE__, #c);  \
      fprintf(stderr, __VA_ARGS__);                                 \
      fprintf(stderr, " (%s)\n", kv_last_error());                  \
      ++g_fail;                                                     \
    }                                                               \
  } while (0)
#define HIP_OK(e)                                                                  \
  do {                                                                             \
    hipError_t e_ = (e);                                                           \
    if (e_ != hipSuccess) {                                                        \
      fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      return 2;                                                                    \
    }                                                                              \
  } while (0)

static inline uint8_t pattern(int p, int b, int64_t off) {
  uint32_t x = (uint32_t)p * 2654435761u ^ (uint32_t)b * 40503u ^ (uint32_t)off * 2246822519u;
  x ^= x >> 15;
  return (uint8_t)(x * 31u >> 7);
}

int main() {
  const int L = 3, H = 2, D = 64, B = 16, E = 2, N = 96;
  const int P = 2 * L;
  const int64_t C = (int64_t)B * H * D * E;  // 4 KiB
  const int64_t R = P * C;
  std::vector<uint8_t> pool_host((size_t)(P * N * C));
  for (int p = 0; p < P; ++p)
    for (int b = 0; b < N; ++b)
      for (int64_t o = 0; o < C; ++o) pool_host[(size_t)(((int64_t)p * N + b) * C + o)] = pattern(p, b, o);
  void* gpu = nullptr;
  HIP_OK(hipMalloc(&gpu, pool_host.size()));
  HIP_OK(hipMemcpy(gpu, pool_host.data(), pool_host.size(), hipMemcpyHostToDevice));

  kv_pool_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L, cfg.n_kv_heads = H, cfg.head_dim = D, cfg.block_size = B, cfg.elt_bytes = E;
  cfg.n_gpu_blocks = N;
  cfg.gpu_base = gpu;
  cfg.host_bytes = 80 * R;
  cfg.host_slack_blocks = 2;
  kv_pool_t* pool = nullptr;
  EXPECT(kv_pool_create(&cfg, &pool) == KV_OK, "create");
  if (!pool) return 1;
  int64_t rb = 0;
  EXPECT(kv_record_bytes(pool, &rb) == KV_OK && rb == R, "record bytes %lld", (long long)rb);

  // request 1: 20 blocks through a permuted table; request 2 right behind it in the arena
  std::vector<int32_t> t1, t2;
  for (int j = 0; j < 20; ++j) t1.push_back((j * 37 + 5) % N);
  for (int j = 0; j < 10; ++j) t2.push_back((j * 41 + 11) % N);
  EXPECT(swap_out(pool, 1, t1.data(), 20) == KV_OK, "swap_out 1");
  EXPECT(swap_out(pool, 2, t2.data(), 10) == KV_OK, "swap_out 2");

  auto check = [&](int64_t req, const std::vector<int32_t>& table, int first, int n, const uint8_t* got) {
    for (int j = 0; j < n; ++j)
      for (int p = 0; p < P; ++p)
        for (int64_t o = 0; o < C; ++o) {
          const uint8_t want = pattern(p, table[(size_t)(first + j)], o);
          const uint8_t have = got[((int64_t)j * P + p) * C + o];
          if (want != have) {
            EXPECT(false, "req %lld block %d plane %d offset %lld: %u != %u", (long long)req, first + j, p,
                   (long long)o, have, want);
            return;
          }
        }
  };

  std::vector<uint8_t> buf((size_t)(40 * R), 0xEE);
  // no explicit wait: kv_host_read waits for the request's last op itself
  EXPECT(kv_host_read(pool, 1, 0, 20, buf.data()) == KV_OK, "read whole image");
  check(1, t1, 0, 20, buf.data());
  EXPECT(buf[(size_t)(20 * R)] == 0xEE, "wrote past the end");
  EXPECT(kv_host_read(pool, 1, 7, 5, buf.data()) == KV_OK, "read a window");
  check(1, t1, 7, 5, buf.data());
  const void* view = nullptr;
  int64_t bytes = 0;
  EXPECT(kv_host_view(pool, 1, &view, &bytes) == KV_OK && view && bytes == 20 * R, "view of a one-extent image");
  if (view) check(1, t1, 0, 20, (const uint8_t*)view);

  // grow request 1 past its slack: request 2 sits behind it, so the image gets a second extent
  for (int j = 20; j < 31; ++j) t1.push_back((j * 37 + 5) % N);
  std::vector<uint8_t> dirty(31, 0);
  for (int j = 20; j < 31; ++j) dirty[(size_t)j] = 1;
  int32_t moved = 0;
  EXPECT(swap_out_delta(pool, 1, t1.data(), 31, dirty.data(), &moved) == KV_OK && moved == 11, "delta moved %d", moved);
  int32_t n_img = 0, n_ext = 0;
  EXPECT(kv_host_len(pool, 1, &n_img, &n_ext) == KV_OK && n_img == 31 && n_ext == 2, "image %d blocks in %d extents", n_img, n_ext);
  EXPECT(kv_host_view(pool, 1, &view, &bytes) == KV_OK && view == nullptr && bytes == 31 * R, "no zero-copy view of two extents");
  EXPECT(kv_host_read(pool, 1, 0, 31, buf.data()) == KV_OK, "read across extents");
  check(1, t1, 0, 31, buf.data());
  EXPECT(kv_host_read(pool, 1, 18, 8, buf.data()) == KV_OK, "read a window across the extent boundary");
  check(1, t1, 18, 8, buf.data());

  // errors
  EXPECT(kv_host_read(pool, 1, 30, 2, buf.data()) == KV_EINVAL, "window past the end");
  EXPECT(kv_host_read(pool, 99, 0, 1, buf.data()) == KV_ENOENT, "unknown request");
  EXPECT(kv_host_read(pool, 1, 0, 1, nullptr) == KV_EINVAL, "null destination");

  EXPECT(kv_pool_destroy(pool) == KV_OK, "destroy");
  HIP_OK(hipFree(gpu));
  printf("host_read_check: %d failures\n", g_fail);
  return g_fail ? 1 : 0;
}
