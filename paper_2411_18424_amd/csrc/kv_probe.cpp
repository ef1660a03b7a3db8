// Bandwidth probes of the KV-swap library: the measured host-link peak and the device copy
// ceiling that swaps are compared with.

#include "kv_pool.hpp"

using namespace kvi;

extern "C" {

int32_t kv_link_probe(int64_t bytes, int32_t direction, int32_t reps, double* out_gbps) {
  if (bytes <= 0 || direction < 0 || direction > 2 || reps <= 0 || !out_gbps) return fail(KV_EINVAL, "bad argument");
  void *h0 = nullptr, *h1 = nullptr, *d0 = nullptr, *d1 = nullptr;
  hipStream_t s0 = nullptr, s1 = nullptr;
  int32_t rc = KV_OK;
  double best = 0.0;
  auto cleanup = [&]() {
    if (s0) (void)hipStreamDestroy(s0);
    if (s1) (void)hipStreamDestroy(s1);
    if (h0) (void)hipHostFree(h0);
    if (h1) (void)hipHostFree(h1);
    if (d0) (void)hipFree(d0);
    if (d1) (void)hipFree(d1);
  };
#define PROBE_TRY(expr)                                                      \
  do {                                                                       \
    hipError_t e_ = (expr);                                                  \
    if (e_ != hipSuccess) {                                                  \
      rc = fail(KV_EHIP, "%s: %s", #expr, hipGetErrorString(e_));            \
      cleanup();                                                             \
      return rc;                                                             \
    }                                                                        \
  } while (0)
  PROBE_TRY(hipStreamCreateWithFlags(&s0, hipStreamNonBlocking));
  PROBE_TRY(hipStreamCreateWithFlags(&s1, hipStreamNonBlocking));
  PROBE_TRY(hipHostMalloc(&h0, (size_t)bytes, hipHostMallocDefault));
  PROBE_TRY(hipMalloc(&d0, (size_t)bytes));
  memset(h0, 1, (size_t)bytes);
  if (direction == 2) {
    PROBE_TRY(hipHostMalloc(&h1, (size_t)bytes, hipHostMallocDefault));
    PROBE_TRY(hipMalloc(&d1, (size_t)bytes));
    memset(h1, 2, (size_t)bytes);
  }
  // Each stream carries copies of one direction only, from its very first copy on (the first
  // repetition below is the warm-up): a stream that has carried both directions shared a copy
  // engine with the other stream in the two-way measurement, which then read 60 GB/s instead of 100.
  PROBE_TRY(hipMemsetAsync(d0, 3, (size_t)bytes, s0));  // a fill kernel, not a copy
  PROBE_TRY(hipStreamSynchronize(s0));
  for (int r = 0; r < reps + 1; ++r) {
    auto t0 = std::chrono::steady_clock::now();
    if (direction == 0 || direction == 2) PROBE_TRY(hipMemcpyAsync(h0, d0, (size_t)bytes, hipMemcpyDeviceToHost, s0));
    if (direction == 1) PROBE_TRY(hipMemcpyAsync(d0, h0, (size_t)bytes, hipMemcpyHostToDevice, s0));
    if (direction == 2) PROBE_TRY(hipMemcpyAsync(d1, h1, (size_t)bytes, hipMemcpyHostToDevice, s1));
    PROBE_TRY(hipStreamSynchronize(s0));
    PROBE_TRY(hipStreamSynchronize(s1));
    double sec = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    double gbps = (direction == 2 ? 2.0 : 1.0) * (double)bytes / sec / 1e9;
    if (r > 0 && gbps > best) best = gbps;  // first repetition is warm-up
  }
  cleanup();
  *out_gbps = best;
  return KV_OK;
#undef PROBE_TRY
}

int32_t kv_hbm_probe(int64_t bytes, int32_t reps, double* out_gbps) {
  if (bytes <= 0 || (bytes & 15) || reps <= 0 || !out_gbps) return fail(KV_EINVAL, "bad argument");
  void *a = nullptr, *b = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipStream_t s = nullptr;
  int32_t rc = KV_OK;
  double best = 0.0;
  auto cleanup = [&]() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (s) (void)hipStreamDestroy(s);
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
  };
#define PROBE_TRY(expr)                                                      \
  do {                                                                       \
    hipError_t e_ = (expr);                                                  \
    if (e_ != hipSuccess) {                                                  \
      rc = fail(KV_EHIP, "%s: %s", #expr, hipGetErrorString(e_));            \
      cleanup();                                                             \
      return rc;                                                             \
    }                                                                        \
  } while (0)
  PROBE_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
  PROBE_TRY(hipMalloc(&a, (size_t)bytes));
  PROBE_TRY(hipMalloc(&b, (size_t)bytes));
  PROBE_TRY(hipMemsetAsync(a, 1, (size_t)bytes, s));
  PROBE_TRY(hipEventCreate(&e0));
  PROBE_TRY(hipEventCreate(&e1));
  for (int r = 0; r < reps + 1; ++r) {
    PROBE_TRY(kv_launch_linear_copy(b, a, bytes, s, e0, e1));
    PROBE_TRY(hipStreamSynchronize(s));
    float ms = 0.f;
    PROBE_TRY(hipEventElapsedTime(&ms, e0, e1));
    double gbps = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
    if (r > 0 && gbps > best) best = gbps;
  }
  cleanup();
  *out_gbps = best;
  return KV_OK;
#undef PROBE_TRY
}

}  // extern "C"
