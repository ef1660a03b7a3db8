// Host-logic stress of the KV-swap library through its C ABI, in a plan-only pool (no HIP
// call is made, no GPU is needed): several threads drive swaps, the reuse map, both
// allocators and a swap manager at once.  Built with the host sanitizers by
// tests/test_host_sanitizers.py; every status must be one the header allows for the call,
// and at the end everything must have been given back.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <thread>
#include <vector>

#include "../../include/kvswap.h"

static std::atomic<int> g_failures{0};

#define EXPECT(cond, ...)                      \
  do {                                         \
    if (!(cond)) {                             \
      fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
      fprintf(stderr, __VA_ARGS__);            \
      fprintf(stderr, " (%s)\n", kv_last_error()); \
      g_failures++;                            \
    }                                          \
  } while (0)

static uint64_t mix(uint64_t* s) {  // splitmix64
  uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static const int N_BLOCKS = 512;
static const int REQS_PER_THREAD = 8;

static bool one_of(int32_t rc, std::initializer_list<int32_t> ok) {
  for (int32_t v : ok)
    if (rc == v) return true;
  return false;
}

// A serving loop of its own requests: tables come from the shared allocator.
static void swapper(kv_pool_t* pool, int tid, int iters) {
  uint64_t rng = 1000 + (uint64_t)tid;
  struct Req {
    std::vector<int32_t> table;
    bool has_image = false;
    int32_t image_len = 0;
  } reqs[REQS_PER_THREAD];
  const int64_t base = (int64_t)tid * 100;
  for (int it = 0; it < iters; ++it) {
    Req& q = reqs[mix(&rng) % REQS_PER_THREAD];
    const int64_t id = base + (&q - reqs);
    switch (mix(&rng) % 8) {
      case 0:
      case 1: {  // (re)start or grow
        int32_t extra = 1 + (int32_t)(mix(&rng) % 12);
        std::vector<int32_t> ids((size_t)extra);
        int32_t runs = 0;
        int32_t rc = alloc_block_group(pool, id, extra, 4, ids.data(), &runs);
        EXPECT(one_of(rc, {KV_OK, KV_ENOMEM_GPU}), "alloc_block_group -> %d", rc);
        if (rc == KV_OK) {
          EXPECT(runs >= 1 && runs <= extra, "runs %d of %d", runs, extra);
          q.table.insert(q.table.end(), ids.begin(), ids.end());
        }
        break;
      }
      case 2: {  // preempt: delta when there is an image
        if (q.table.empty()) break;
        int32_t n = (int32_t)q.table.size();
        int32_t rc;
        if (q.has_image && n >= q.image_len) {
          std::vector<uint8_t> dirty((size_t)n);
          for (auto& d : dirty) d = mix(&rng) % 4 == 0;
          int32_t moved = -1;
          rc = swap_out_delta(pool, id, q.table.data(), n, dirty.data(), &moved);
          EXPECT(one_of(rc, {KV_OK, KV_ENOMEM_HOST}), "swap_out_delta -> %d", rc);
          if (rc == KV_OK) EXPECT(moved >= n - q.image_len && moved <= n, "moved %d of %d", moved, n);
        } else {
          rc = swap_out(pool, id, q.table.data(), n);
          EXPECT(one_of(rc, {KV_OK, KV_ENOMEM_HOST}), "swap_out -> %d", rc);
        }
        if (rc == KV_OK) {
          q.has_image = true;
          q.image_len = n;
          rc = free_block_group(pool, id, q.table.data(), n);
          EXPECT(rc == KV_OK, "free_block_group -> %d", rc);
          q.table.clear();
        }
        break;
      }
      case 3: {  // resume
        if (!q.table.empty() || !q.has_image || q.image_len == 0) break;
        std::vector<int32_t> ids((size_t)q.image_len);
        int32_t rc = alloc_block_group(pool, id, q.image_len, 1, ids.data(), nullptr);
        EXPECT(one_of(rc, {KV_OK, KV_ENOMEM_GPU}), "alloc_block_group -> %d", rc);
        if (rc != KV_OK) break;
        if (mix(&rng) % 2)
          rc = swap_in(pool, id, ids.data(), q.image_len);
        else
          rc = swap_in_layerwise(pool, id, ids.data(), q.image_len, nullptr, 1 + (int32_t)(mix(&rng) % 2), nullptr);
        // a contaminated image cannot come back whole
        EXPECT(one_of(rc, {KV_OK, KV_ENOENT}), "swap_in -> %d", rc);
        if (rc == KV_OK) {
          q.table = ids;
        } else {
          EXPECT(free_block_group(pool, id, ids.data(), q.image_len) == KV_OK, "free after refused swap_in");
          EXPECT(kv_host_release(pool, id) == KV_OK, "release");
          q.has_image = false;
        }
        break;
      }
      case 4: {  // contamination of a running request's copy
        if (!q.has_image || q.table.empty() || q.image_len == 0) break;
        std::vector<uint8_t> mask((size_t)q.image_len);
        for (auto& m : mask) m = mix(&rng) % 3 == 0;
        EXPECT(kv_host_invalidate(pool, id, mask.data(), q.image_len) == KV_OK, "invalidate");
        break;
      }
      case 5: {  // completion calls
        int32_t done = -1;
        int32_t rc = kv_query(pool, id, &done);
        EXPECT(one_of(rc, {KV_OK, KV_ENOENT}), "kv_query -> %d", rc);
        if (rc == KV_OK) EXPECT(done == 1, "plan-only work is done at once");
        rc = kv_wait(pool, id);
        EXPECT(one_of(rc, {KV_OK, KV_ENOENT}), "kv_wait -> %d", rc);
        rc = kv_wait_layer(pool, id, 1);
        EXPECT(one_of(rc, {KV_OK, KV_ENOENT}), "kv_wait_layer -> %d", rc);
        break;
      }
      case 6: {  // finish
        if (!q.table.empty()) {
          EXPECT(free_block_group(pool, id, q.table.data(), (int32_t)q.table.size()) == KV_OK, "free");
          q.table.clear();
        }
        if (q.has_image) {
          EXPECT(kv_host_release(pool, id) == KV_OK, "release");
          q.has_image = false;
        }
        break;
      }
      default: {  // bad calls must be refused without effect
        int32_t bad[3] = {0, 0, N_BLOCKS};
        EXPECT(swap_out(pool, id + 50, bad, 2) == KV_EINVAL, "duplicate ids accepted");
        EXPECT(swap_out(pool, id + 50, bad + 1, 2) == KV_EINVAL, "out-of-range id accepted");
        EXPECT(swap_in(pool, id + 50, bad, 1) == KV_ENOENT, "swap_in without image accepted");
        EXPECT(strstr(kv_last_error(), "no host copy") != nullptr, "error text is per thread");
        break;
      }
    }
  }
  for (Req& q : reqs) {
    const int64_t id = base + (&q - reqs);
    if (!q.table.empty())
      EXPECT(free_block_group(pool, id, q.table.data(), (int32_t)q.table.size()) == KV_OK, "final free");
    if (q.has_image) EXPECT(kv_host_release(pool, id) == KV_OK, "final release");
  }
}

// Requests that grow through the block-group manager.
static void grower(kv_pool_t* pool, int tid, int iters) {
  uint64_t rng = 5000 + (uint64_t)tid;
  const int64_t base = 10000 + (int64_t)tid * 100;
  bool open[4] = {false, false, false, false};
  for (int it = 0; it < iters; ++it) {
    int r = (int)(mix(&rng) % 4);
    if (mix(&rng) % 5 == 0) {
      if (open[r]) {
        EXPECT(kv_bg_close(pool, base + r) == KV_OK, "kv_bg_close");
        open[r] = false;
      }
      continue;
    }
    int32_t n = 1 + (int32_t)(mix(&rng) % 6);
    std::vector<int32_t> ids((size_t)n);
    int32_t rc = kv_bg_append(pool, base + r, n, 2, ids.data());
    EXPECT(one_of(rc, {KV_OK, KV_ENOMEM_GPU}), "kv_bg_append -> %d", rc);
    if (rc == KV_OK) {
      open[r] = true;
      for (int32_t b : ids) EXPECT(b >= 0 && b < N_BLOCKS, "id %d", b);
      int32_t len = 0;
      std::vector<int32_t> table(4096);
      EXPECT(kv_bg_table(pool, base + r, table.data(), 4096, &len) == KV_OK && len >= n, "kv_bg_table");
    }
  }
  for (int r = 0; r < 4; ++r)
    if (open[r]) EXPECT(kv_bg_close(pool, base + r) == KV_OK, "final kv_bg_close");
}

// A scheduler thread that hands its swaps to the swap manager.
static void scheduler(kv_pool_t* pool, int iters) {
  kv_manager_t* mgr = nullptr;
  EXPECT(kv_manager_create(pool, nullptr, &mgr) == KV_OK, "kv_manager_create");
  if (!mgr) return;
  uint64_t rng = 77;
  const int64_t base = 20000;
  std::vector<int32_t> table(16);
  int32_t rc = alloc_block_group(pool, base, 16, 1, table.data(), nullptr);
  EXPECT(rc == KV_OK, "scheduler alloc -> %d", rc);
  uint64_t submitted = 0, reported = 0;
  for (int it = 0; it < iters && rc == KV_OK; ++it) {
    uint64_t t1 = 0, t2 = 0;
    EXPECT(kv_manager_submit(mgr, KV_TASK_SWAP_OUT, base, table.data(), 16, nullptr, &t1) == KV_OK, "submit out");
    EXPECT(kv_manager_submit(mgr, KV_TASK_SWAP_IN, base, table.data(), 16, nullptr, &t2) == KV_OK, "submit in");
    submitted += 2;
    if (mix(&rng) % 3 == 0) {
      int32_t st = -99;
      EXPECT(kv_manager_wait(mgr, t2, &st) == KV_OK && st == KV_OK, "wait -> status %d", st);
      reported += 1;
    }
    uint64_t tickets[8];
    int32_t status[8], n = 0;
    EXPECT(kv_manager_poll(mgr, tickets, status, 8, &n) == KV_OK, "poll");
    for (int i = 0; i < n; ++i) EXPECT(status[i] == KV_OK, "task status %d", status[i]);
    reported += (uint64_t)n;
    int32_t async = -1;
    EXPECT(kv_manager_strategy(mgr, 1, 16, &async) == KV_OK && (async == 0 || async == 1), "strategy");
  }
  EXPECT(kv_manager_drain(mgr) == KV_OK, "drain");
  for (;;) {
    uint64_t tickets[8];
    int32_t n = 0;
    EXPECT(kv_manager_poll(mgr, tickets, nullptr, 8, &n) == KV_OK, "poll");
    if (n == 0) break;
    reported += (uint64_t)n;
  }
  EXPECT(reported == submitted, "each task reported once: %llu of %llu", (unsigned long long)reported,
         (unsigned long long)submitted);
  kv_manager_stats_t ms;
  EXPECT(kv_manager_stats(mgr, &ms) == KV_OK && ms.dispatched == (int64_t)submitted && ms.failed == 0, "manager stats");
  EXPECT(kv_manager_destroy(mgr) == KV_OK, "kv_manager_destroy");
  if (rc == KV_OK) {
    EXPECT(free_block_group(pool, base, table.data(), 16) == KV_OK, "scheduler free");
    EXPECT(kv_host_release(pool, base) == KV_OK, "scheduler release");
  }
}

// A scheduler thread that runs Algorithm 1 through kv_manager_iterate: two requests take turns,
// one leaves while the other resumes into the blocks it vacates (a conflict in every iteration).
static void iterating_scheduler(kv_pool_t* pool, int iters) {
  kv_manager_t* mgr = nullptr;
  EXPECT(kv_manager_create(pool, nullptr, &mgr) == KV_OK, "kv_manager_create");
  if (!mgr) return;
  const int64_t a = 30000, b = 30001;
  std::vector<int32_t> table(12);
  int32_t rc = alloc_block_group(pool, a, 12, 1, table.data(), nullptr);
  EXPECT(rc == KV_OK, "iterating scheduler alloc -> %d", rc);
  if (rc != KV_OK) {
    kv_manager_destroy(mgr);
    return;
  }
  EXPECT(kv_host_set_priority(pool, a, 100) == KV_OK && kv_host_set_priority(pool, b, 100) == KV_OK, "priority");
  int32_t twelve = 12, n_res = 0;
  int64_t resumed[4];
  kv_iteration_t it;
  memset(&it, 0, sizeof it);
  it.n_swap_out = 1, it.out_reqs = &b, it.out_tables = table.data(), it.out_n_blocks = &twelve;
  EXPECT(kv_manager_iterate(mgr, &it, resumed, 4, &n_res, nullptr) == KV_OK && n_res == 0, "first iterate");
  int64_t out = a, in = b, total_resumed = 0, swap_ins = 0;
  for (int k = 0; k < iters; ++k) {
    int32_t where = -1;
    EXPECT(kv_manager_where(mgr, in, &where) == KV_OK, "where");
    if (where != KV_WHERE_SWAPPED || (kv_manager_where(mgr, out, &where) == KV_OK && where != KV_WHERE_RUNNING)) {
      memset(&it, 0, sizeof it);  // an asynchronous swap-in is still ongoing: poll
      EXPECT(kv_manager_iterate(mgr, &it, resumed, 4, &n_res, nullptr) == KV_OK, "polling iterate");
      total_resumed += n_res;
      continue;
    }
    memset(&it, 0, sizeof it);
    it.n_swap_in = 1, it.in_reqs = &in, it.in_tables = table.data(), it.in_n_blocks = &twelve;
    it.n_swap_out = 1, it.out_reqs = &out, it.out_tables = table.data(), it.out_n_blocks = &twelve;
    it.force_mode = 1 + k % 2;
    kv_iteration_result_t res;
    rc = kv_manager_iterate(mgr, &it, resumed, 4, &n_res, &res);
    EXPECT(rc == KV_OK && res.conflicts == 1, "iterate -> %d, conflicts %d", rc, res.conflicts);
    total_resumed += n_res;
    ++swap_ins;
    std::swap(out, in);
  }
  EXPECT(kv_manager_drain(mgr) == KV_OK, "drain");
  memset(&it, 0, sizeof it);
  EXPECT(kv_manager_iterate(mgr, &it, resumed, 4, &n_res, nullptr) == KV_OK, "last iterate");
  total_resumed += n_res;
  int64_t fr[4];
  int32_t fs[4], nf = 0;
  EXPECT(kv_manager_failures(mgr, fr, fs, 4, &nf) == KV_OK, "failures");
  // the tight arena may refuse a swap-out (priority protects these two from eviction, not from a full arena)
  EXPECT(total_resumed + nf >= swap_ins - 1 && total_resumed <= swap_ins, "resumed %lld of %lld swap-ins, %d failures",
         (long long)total_resumed, (long long)swap_ins, nf);
  EXPECT(kv_manager_destroy(mgr) == KV_OK, "kv_manager_destroy");
  EXPECT(free_block_group(pool, a, table.data(), 12) == KV_OK, "iterating scheduler free");
  (void)kv_host_release(pool, a);
  (void)kv_host_release(pool, b);
}

// Readers of global state.
static void observer(kv_pool_t* pool, std::atomic<bool>* stop) {
  while (!stop->load()) {
    kv_stats_t st;
    EXPECT(kv_stats(pool, &st) == KV_OK, "kv_stats");
    EXPECT(st.host_arena_used >= 0 && st.host_arena_used <= st.host_arena_bytes, "arena accounting");
    int64_t free_blocks = -1, largest = -1;
    EXPECT(kv_free_blocks(pool, &free_blocks, &largest) == KV_OK, "kv_free_blocks");
    EXPECT(free_blocks >= 0 && free_blocks <= N_BLOCKS && largest <= free_blocks, "free %lld largest %lld",
           (long long)free_blocks, (long long)largest);
    EXPECT(kv_wait_all(pool) == KV_OK, "kv_wait_all");
    std::this_thread::yield();
  }
}

int main(int argc, char** argv) {
  const int iters = argc > 1 ? atoi(argv[1]) : 20000;
  kv_pool_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 2;
  cfg.n_kv_heads = 4;
  cfg.head_dim = 64;
  cfg.block_size = 16;
  cfg.elt_bytes = 2;  // C = 8 KiB, R = 32 KiB
  cfg.flags = KV_FLAG_PLAN_ONLY | KV_FLAG_HOST_EVICT;
  cfg.n_gpu_blocks = N_BLOCKS;
  cfg.host_bytes = 300 * 32768;  // tight: eviction and refusals happen
  cfg.host_slack_blocks = 3;
  kv_pool_t* pool = nullptr;
  if (kv_pool_create(&cfg, &pool) != KV_OK) {
    fprintf(stderr, "kv_pool_create: %s\n", kv_last_error());
    return 2;
  }
  EXPECT(kv_bg_configure(pool, 8, 42) == KV_OK, "kv_bg_configure");
  std::atomic<bool> stop{false};
  std::vector<std::thread> th;
  for (int t = 0; t < 3; ++t) th.emplace_back(swapper, pool, t, iters);
  for (int t = 0; t < 2; ++t) th.emplace_back(grower, pool, t, iters);
  th.emplace_back(scheduler, pool, iters / 10);
  th.emplace_back(iterating_scheduler, pool, iters / 10);
  std::thread obs(observer, pool, &stop);
  for (auto& t : th) t.join();
  stop = true;
  obs.join();
  kv_stats_t st;
  EXPECT(kv_stats(pool, &st) == KV_OK && st.host_arena_used == 0, "host arena not given back: %lld bytes",
         (long long)st.host_arena_used);
  int64_t free_blocks = 0, largest = 0;
  EXPECT(kv_free_blocks(pool, &free_blocks, &largest) == KV_OK && free_blocks == N_BLOCKS && largest == N_BLOCKS,
         "GPU blocks not given back: %lld free, largest run %lld", (long long)free_blocks, (long long)largest);
  EXPECT(kv_pool_destroy(pool) == KV_OK, "kv_pool_destroy");
  printf("plan_stress: %d failures, %lld blocks out, %lld blocks in, %lld evicted\n", g_failures.load(),
         (long long)st.blocks_out, (long long)st.blocks_in, (long long)st.host_evicted_blocks);
  return g_failures.load() ? 1 : 0;
}
