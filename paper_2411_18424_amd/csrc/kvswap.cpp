// C ABI of the KV-swap library: pool creation and destruction, and the entry points declared
// in include/kvswap.h.  The copy engine is in kv_engine.cpp, validation / host images / moved-
// set selection in kv_reuse.cpp, the allocators in kv_alloc.hpp, the kernels in kv_kernels.hip,
// the swap manager in kv_manager.cpp.
//
// FastSwitch (arXiv 2411.18424) swaps a preempted request's KV cache to CPU memory and
// back (Section 2.1), wants large transfers instead of one small copy per block (Section
// 2.2 Challenge #1, Section 3.1), overlaps swapping with inference and resolves conflicts
// between blocks of in-flight swaps and newly allocated blocks (Section 3.2), and reuses
// the CPU copy across conversation turns (Section 3.3).  On MI355X the transfer scheme is
// a pack kernel plus few large pinned copies rather than one copy per block group: HBM is
// two orders of magnitude faster than the host link, so the extra pass is nearly free and
// the copy size no longer depends on fragmentation.
//
// Streams (all default priority, non-blocking): one per direction by default (gathers and
// device-to-host copies on one, host-to-device copies and scatters on the other); with
// KV_FLAG_FOUR_STREAMS kernels and copies of each direction get streams of their own:
//   s_pack : gather kernels           s_d2h : device-to-host copies
//   s_h2d  : host-to-device copies    s_scat: scatter kernels

#include "kv_pool.hpp"

namespace kvi {

thread_local std::string g_err;

int32_t fail(int32_t code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

}  // namespace kvi

using namespace kvi;

namespace {

void destroy_pool(kv_pool* p) {
  {
    std::unique_lock<std::mutex> lk(p->mu);
    stop_copy_thread(p, lk);  // after it has enqueued what it holds
  }
  if (!p->plan) {
    // wait for the library's own streams only: the caller's streams are none of its business
    for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat})
      if (s) (void)hipStreamSynchronize(s);
    for (ByteRing* r : {&p->ring_out, &p->ring_in})
      for (Region& g : r->live)
        if (g.freed) (void)hipEventDestroy(g.freed);
    for (auto* dq : {&p->ops_out, &p->ops_in})
      for (auto& o : *dq) {
        if (o->packed) (void)hipEventDestroy(o->packed);
        if (o->done) (void)hipEventDestroy(o->done);
        for (hipEvent_t e : o->aux) (void)hipEventDestroy(e);
        for (hipEvent_t e : o->timed) (void)hipEventDestroy(e);
        for (hipEvent_t e : o->layer_ev)
          if (e) (void)hipEventDestroy(e);
      }
    for (hipEvent_t e : p->event_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->timing_pool) (void)hipEventDestroy(e);
    for (auto& r : p->prof) {
      (void)hipEventDestroy(r.start);
      (void)hipEventDestroy(r.stop);
    }
    if (p->ev_compute) (void)hipEventDestroy(p->ev_compute);
    if (p->s_d2h == p->s_pack) p->s_d2h = nullptr;  // aliases of the other two
    if (p->s_scat == p->s_h2d) p->s_scat = nullptr;
    for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat})
      if (s) (void)hipStreamDestroy(s);
    if (p->own_staging && p->staging) (void)hipFree(p->staging);
    if (p->host) (void)hipHostFree(p->host);
  }
  delete p;
}

}  // namespace

// =============================================================== C ABI
extern "C" {

const char* kv_last_error(void) { return g_err.c_str(); }
const char* kv_version(void) { return "kvswap 0.1 (gfx950)"; }

int32_t kv_pool_create(const kv_pool_config_t* cfg, kv_pool_t** out) {
  if (!cfg || !out) return fail(KV_EINVAL, "null argument");
  if (cfg->n_layers <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0 || cfg->block_size <= 0 ||
      cfg->elt_bytes <= 0 || cfg->n_gpu_blocks <= 0)
    return fail(KV_EINVAL, "shape fields must be positive");
  if (cfg->n_gpu_blocks > 0x7FFFFFFFll) return fail(KV_EINVAL, "block ids are int32");
  const int64_t C = (int64_t)cfg->block_size * cfg->n_kv_heads * cfg->head_dim * cfg->elt_bytes;
  if (C % 16 != 0 || C > 0x7FFFFFF0ll) return fail(KV_EINVAL, "chunk size %lld must be a multiple of 16 bytes", (long long)C);
  const bool plan = (cfg->flags & KV_FLAG_PLAN_ONLY) != 0;
  if (!plan && (!cfg->gpu_base || ((uintptr_t)cfg->gpu_base & 15)))
    return fail(KV_EINVAL, "gpu_base must be a 16-byte aligned device pointer");
  if (cfg->staging_base && ((uintptr_t)cfg->staging_base & 15))
    return fail(KV_EINVAL, "staging_base must be 16-byte aligned");
  if (cfg->host_bytes < 0 || cfg->staging_out_bytes < 0 || cfg->staging_in_bytes < 0 ||
      cfg->max_piece_bytes < 0 || cfg->copy_chunk_bytes < 0)
    return fail(KV_EINVAL, "negative size");
  if (cfg->mapped_out_max_blocks < 0) return fail(KV_EINVAL, "negative mapped_out_max_blocks");
  if (cfg->defer_min_bytes < 0) return fail(KV_EINVAL, "negative defer_min_bytes");

  kv_pool* p = new kv_pool();
  p->cfg = *cfg;
  p->plan = plan;
  p->profile = (cfg->flags & KV_FLAG_PROFILE) != 0 && !plan;
  p->order_compute = (cfg->flags & KV_FLAG_ORDER_COMPUTE) != 0;
  p->N = cfg->n_gpu_blocks;
  p->C = C;
  p->P = 2 * cfg->n_layers;
  p->R = p->P * C;
  p->gpu = (char*)cfg->gpu_base;
  p->compute = (hipStream_t)cfg->compute_stream;
  p->slack = cfg->host_slack_blocks < 0 ? 32 : cfg->host_slack_blocks;
  p->copy_chunk = cfg->copy_chunk_bytes > 0 ? cfg->copy_chunk_bytes : (256ll << 20);
  p->grid = cfg->gather_grid;
  p->unroll = cfg->tile_unroll;  // 0 = pick from the chunk size
  p->variant = cfg->pack_variant;
  p->mapped_in = (cfg->flags & KV_FLAG_MAPPED_SWAP_IN) != 0;
  p->host_evict = (cfg->flags & KV_FLAG_HOST_EVICT) != 0;
  p->mapped_out = (cfg->flags & KV_FLAG_MAPPED_SWAP_OUT) != 0;
  p->mapped_out_max = cfg->mapped_out_max_blocks;
  p->strided_copies = (cfg->flags & KV_FLAG_NO_STRIDED_COPIES) == 0;
  p->defer_copies = (cfg->flags & KV_FLAG_NO_DEFER_COPIES) == 0;
  p->defer_min = cfg->defer_min_bytes > 0 ? cfg->defer_min_bytes : (16ll << 20);
  p->second_lane = (cfg->flags & KV_FLAG_SECOND_LANE) != 0;
  p->launch_events = (cfg->flags & KV_FLAG_NO_LAUNCH_EVENTS) == 0;
  if (cfg->mapped_in_grid > 0) p->mapped_grid = cfg->mapped_in_grid;
  p->launch_blocks = kv_max_launch_blocks((uint32_t)C, (uint32_t)p->P, p->unroll, p->variant);
  // staging rings: defaults scale with the pool, capped at 4 GiB (out) and 1 GiB (in)
  const int64_t pool_bytes = p->R * p->N;
  auto round_R = [&](int64_t b) { return b / p->R * p->R; };
  int64_t out_cap = cfg->staging_out_bytes > 0
                        ? cfg->staging_out_bytes
                        : std::min<int64_t>(4ll << 30, std::max<int64_t>(2 * p->R, pool_bytes / 4));
  int64_t in_cap = cfg->staging_in_bytes > 0
                       ? cfg->staging_in_bytes
                       : std::min<int64_t>(1ll << 30, std::max<int64_t>(2 * p->R, pool_bytes / 8));
  out_cap = round_R(out_cap);
  in_cap = round_R(in_cap);
  if (out_cap < 2 * p->R || in_cap < 2 * p->R) {
    delete p;
    return fail(KV_EINVAL, "staging too small: each ring must hold two block records (%lld bytes)", (long long)(2 * p->R));
  }
  auto piece_blocks = [&](int64_t cap, int64_t dflt_bytes) {
    int64_t b = cfg->max_piece_bytes > 0 ? cfg->max_piece_bytes : dflt_bytes;
    b = std::min(b, cap / 2);  // two pieces fit, so a large call can pipeline
    return std::max<int64_t>(1, b / p->R);
  };
  p->ring_out.cap = out_cap;
  // four streams: gathers run under the copies, so the first piece is what the link waits for - keep it short
  p->ring_out.piece_blocks = piece_blocks(out_cap, (cfg->flags & KV_FLAG_FOUR_STREAMS) ? (256ll << 20) : p->launch_blocks * p->R);
  p->ring_in.cap = in_cap;
  p->ring_in.piece_blocks = piece_blocks(in_cap, 512ll << 20);
  p->arena_blocks = cfg->host_bytes / p->R;
  if (p->arena_blocks > 0xFFFFFFFFll) {
    delete p;
    return fail(KV_EINVAL, "host arena of %lld records: record indices are 32-bit", (long long)p->arena_blocks);
  }
  p->arena.insert(0, p->arena_blocks);
  p->alloc.init(p->N);
  p->groups.configure(&p->alloc, 64, 20241127);
  p->reader_seq.assign((size_t)p->N, 0);
  p->writer_seq.assign((size_t)p->N, 0);
  p->stamp.assign((size_t)p->N, 0);

  auto bail = [&](int32_t rc) {
    std::string keep = g_err;
    destroy_pool(p);
    g_err = keep;
    return rc;
  };
#define TRY_OR_BAIL(expr)                                                  \
  do {                                                                     \
    hipError_t e_ = (expr);                                                \
    if (e_ != hipSuccess)                                                  \
      return bail(fail(KV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)));  \
  } while (0)

  if (!plan) {
    TRY_OR_BAIL(hipGetDevice(&p->device));
    if (p->grid <= 0) {
      int dev = 0, cus = 256;
      TRY_OR_BAIL(hipGetDevice(&dev));
      TRY_OR_BAIL(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
      p->grid = cus * 8;
    }
    // Side streams.  A process has few hardware queues (4 by default) and streams beyond that
    // share one: a scatter that lands behind the caller's compute kernels on a shared queue
    // waits for all of them.  Two streams (one per direction) are therefore the default;
    // KV_FLAG_FOUR_STREAMS gives kernels and copies of each direction streams of their own,
    // which lets a scatter run under the next piece's copy.
    TRY_OR_BAIL(hipStreamCreateWithFlags(&p->s_pack, hipStreamNonBlocking));
    TRY_OR_BAIL(hipStreamCreateWithFlags(&p->s_h2d, hipStreamNonBlocking));
    if (cfg->flags & KV_FLAG_FOUR_STREAMS) {
      TRY_OR_BAIL(hipStreamCreateWithFlags(&p->s_d2h, hipStreamNonBlocking));
      TRY_OR_BAIL(hipStreamCreateWithFlags(&p->s_scat, hipStreamNonBlocking));
      p->four_streams = true;
    } else {
      p->s_d2h = p->s_pack;
      p->s_scat = p->s_h2d;
      if (cfg->flags & KV_FLAG_SCATTER_STREAM) TRY_OR_BAIL(hipStreamCreateWithFlags(&p->s_scat, hipStreamNonBlocking));
    }
    TRY_OR_BAIL(hipEventCreateWithFlags(&p->ev_compute, hipEventDisableTiming));
    if (p->arena_blocks > 0) {
      hipError_t e = hipHostMalloc((void**)&p->host, (size_t)(p->arena_blocks * p->R), hipHostMallocDefault);
      if (e != hipSuccess) {
        (void)hipGetLastError();  // do not leave the refusal behind for the caller's next runtime call to report
        return bail(fail(KV_ENOMEM_HOST, "hipHostMalloc(%lld): %s", (long long)(p->arena_blocks * p->R), hipGetErrorString(e)));
      }
      TRY_OR_BAIL(hipHostGetDevicePointer((void**)&p->host_dev, p->host, 0));
    }
    if (cfg->staging_base) {
      p->staging = (char*)cfg->staging_base;
    } else {
      hipError_t e = hipMalloc((void**)&p->staging, (size_t)(out_cap + in_cap));
      if (e != hipSuccess) {
        (void)hipGetLastError();
        return bail(fail(KV_ENOMEM_GPU, "hipMalloc(staging %lld): %s", (long long)(out_cap + in_cap), hipGetErrorString(e)));
      }
      p->own_staging = true;
    }
    // address of the static staging array on this device (swap_out_static)
    TRY_OR_BAIL(kv_static_staging(&p->static_staging));
    // The first copies of a process in each direction block the host for milliseconds while
    // the runtime sets its copy paths up: take that here, not inside the first swap.
    if (p->host) {
      const size_t n = (size_t)std::min<int64_t>({1ll << 20, p->arena_blocks * p->R, out_cap + in_cap});
      TRY_OR_BAIL(hipMemcpyAsync(p->staging, p->host, n, hipMemcpyHostToDevice, p->s_h2d));
      TRY_OR_BAIL(hipStreamSynchronize(p->s_h2d));
      TRY_OR_BAIL(hipMemcpyAsync(p->host, p->staging, n, hipMemcpyDeviceToHost, p->s_pack));
      TRY_OR_BAIL(hipStreamSynchronize(p->s_pack));
    }
    // ... and the first kernel launch loads the code object: gather block 0 into staging once
    // (reads the pool, writes only staging).
    {
      KvPackArgs a;
      a.pool = p->gpu;
      a.staging = p->staging;
      a.plane_stride = p->N * p->C;
      a.C = (uint32_t)p->C;
      a.P = (uint32_t)p->P;
      a.m = 1;
      a.tiles_per_chunk = a.n_tiles = a.xcd_blocks = 0;
      a.table[0] = 0;
      TRY_OR_BAIL(kv_launch_pack(false, a, p->unroll, p->variant, p->grid, p->s_pack, nullptr, nullptr));
      TRY_OR_BAIL(hipStreamSynchronize(p->s_pack));
    }
  }
  p->ring_out.base = p->staging;
  p->ring_in.base = p->staging ? p->staging + out_cap : nullptr;
  p->st.host_arena_bytes = p->arena_blocks * p->R;
  *out = p;
  return KV_OK;
#undef TRY_OR_BAIL
}

int32_t kv_pool_destroy(kv_pool_t* p) {
  if (!p) return fail(KV_EINVAL, "null pool");
  destroy_pool(p);
  return KV_OK;
}

// Waits (fine-grained, Section 3.2 conflict handling) for exactly the gathers / scatters that
// still use parked blocks until `need` blocks are free or nothing more can be released.
static int32_t make_free(kv_pool* p, int64_t need) {
  reap(p);
  while (p->alloc.n_free() < need && p->alloc.n_draining() > 0) {
    uint64_t so = 0, si = 0;
    p->alloc.seqs_to_release(std::min(need - p->alloc.n_free(), p->alloc.n_draining()), &so, &si);
    bool waited = false;
    if (!p->plan) {
      Op* o = so ? find_op(p->ops_out, so) : nullptr;
      if (o && o->packed && !o->packed_done) {
        HIP_TRY(hipEventSynchronize(o->packed));
        waited = true;
      }
      Op* w = si ? find_op(p->ops_in, si) : nullptr;
      if (w && w->done && !w->all_done) {
        HIP_TRY(hipEventSynchronize(w->done));
        waited = true;
      }
    }
    if (waited) p->st.conflict_waits++;
    int64_t before = p->alloc.n_draining();
    reap(p);
    if (p->alloc.n_draining() == before) break;
  }
  return KV_OK;
}

int32_t alloc_block_group(kv_pool_t* p, int64_t req, int32_t n_blocks, int32_t min_run,
                          int32_t* out_blocks, int32_t* out_n_runs) {
  (void)req;  // a label for the caller's bookkeeping; ownership is not tracked per request
  if (!p || n_blocks < 0 || min_run < 0 || (n_blocks > 0 && !out_blocks)) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  reap(p);
  if (p->alloc.n_free() < n_blocks) {
    // blocks parked behind unfinished work may cover the shortfall: wait for exactly that work
    if (p->alloc.n_free() + p->alloc.n_draining() < n_blocks)
      return fail(KV_ENOMEM_GPU, "need %d blocks, %lld free", n_blocks,
                  (long long)(p->alloc.n_free() + p->alloc.n_draining()));
    int32_t rc = make_free(p, n_blocks);
    if (rc) return rc;
    if (p->alloc.n_free() < n_blocks) return fail(KV_ENOMEM_GPU, "need %d blocks, %lld free", n_blocks, (long long)p->alloc.n_free());
  }
  std::vector<int32_t> ids;
  ids.reserve((size_t)n_blocks);
  int32_t runs = p->alloc.alloc(n_blocks, &ids, min_run);
  if (n_blocks > 0) memcpy(out_blocks, ids.data(), sizeof(int32_t) * (size_t)n_blocks);
  if (out_n_runs) *out_n_runs = runs;
  return KV_OK;
}

int32_t free_block_group(kv_pool_t* p, int64_t req, const int32_t* blocks, int32_t n_blocks) {
  (void)req;
  if (!p || n_blocks < 0 || (n_blocks > 0 && !blocks)) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  reap(p);
  if (!p->alloc.can_free(blocks, n_blocks, &p->free_stamp, &p->free_epoch))
    return fail(KV_EINVAL, "free of a block that is out of range, repeated, or not allocated");
  p->alloc.free_ids(blocks, n_blocks, p->reader_seq, p->pack_done_seq, p->writer_seq, p->scat_done_seq);
  return KV_OK;
}

int32_t kv_bg_configure(kv_pool_t* p, int32_t first_group_blocks, uint64_t seed) {
  if (!p || first_group_blocks < 0) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  p->groups.configure(&p->alloc, first_group_blocks, seed);
  return KV_OK;
}

int32_t kv_bg_append(kv_pool_t* p, int64_t req, int32_t n_blocks, int32_t reserve_tail, int32_t* out_blocks) {
  if (!p || n_blocks < 0 || reserve_tail < 0 || (n_blocks > 0 && !out_blocks)) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  reap(p);
  if (p->groups.obtainable(req) < n_blocks) {
    int32_t rc = make_free(p, n_blocks);
    if (rc) return rc;
    if (p->groups.obtainable(req) < n_blocks)
      return fail(KV_ENOMEM_GPU, "need %d blocks, %lld obtainable", n_blocks, (long long)p->groups.obtainable(req));
  }
  std::vector<int32_t> ids;
  ids.reserve((size_t)n_blocks);
  p->groups.append(req, n_blocks, reserve_tail, &ids);
  if ((int32_t)ids.size() != n_blocks) return fail(KV_ENOMEM_GPU, "block groups exhausted");
  if (n_blocks > 0) memcpy(out_blocks, ids.data(), sizeof(int32_t) * (size_t)n_blocks);
  return KV_OK;
}

int32_t kv_bg_table(kv_pool_t* p, int64_t req, int32_t* out_blocks, int32_t cap, int32_t* out_n) {
  if (!p || !out_n || cap < 0) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->groups.has(req)) return fail(KV_ENOENT, "request %lld owns no block group", (long long)req);
  std::vector<int32_t> ids;
  p->groups.table(req, &ids);
  *out_n = (int32_t)ids.size();
  if (out_blocks && cap > 0) memcpy(out_blocks, ids.data(), sizeof(int32_t) * (size_t)std::min<int64_t>(cap, (int64_t)ids.size()));
  return KV_OK;
}

int32_t kv_bg_close(kv_pool_t* p, int64_t req) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->groups.has(req)) return fail(KV_ENOENT, "request %lld owns no block group", (long long)req);
  reap(p);
  std::vector<int32_t> ids;
  p->groups.all_blocks(req, &ids);
  p->groups.forget(req);
  p->alloc.free_ids(ids.data(), (int32_t)ids.size(), p->reader_seq, p->pack_done_seq, p->writer_seq, p->scat_done_seq);
  return KV_OK;
}

int32_t kv_bg_stats(kv_pool_t* p, kv_bg_stats_t* out) {
  if (!p || !out) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  const kv::BlockGroupManager::Stats s = p->groups.stats();
  out->n_requests = s.n_requests;
  out->n_groups = s.n_groups;
  out->used_blocks = s.used_blocks;
  out->tail_blocks = s.tail_blocks;
  out->steals = s.steals;
  out->opened = s.opened;
  out->appended_groups = s.appended_groups;
  out->grown_in_place = s.grown_in_place;
  return KV_OK;
}

int32_t kv_free_blocks(kv_pool_t* p, int64_t* out_free, int64_t* out_largest_run) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  reap(p);
  if (out_free) *out_free = p->alloc.n_free() + p->alloc.n_draining();
  if (out_largest_run) *out_largest_run = p->alloc.largest_run();
  return KV_OK;
}

int32_t swap_out(kv_pool_t* p, int64_t req, const int32_t* block_table, int32_t n_blocks) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<OutItem> items(1);
  items[0] = OutItem{req, block_table, n_blocks, nullptr};
  return do_swap_out(p, items, nullptr);
}

int32_t swap_out_delta(kv_pool_t* p, int64_t req, const int32_t* block_table, int32_t n_blocks,
                       const uint8_t* dirty_mask, int32_t* out_n_moved) {
  if (!p) return fail(KV_EINVAL, "null pool");
  if (n_blocks > 0 && !dirty_mask) return fail(KV_EINVAL, "null dirty mask");
  static const uint8_t none = 0;
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<OutItem> items(1);
  items[0] = OutItem{req, block_table, n_blocks, dirty_mask ? dirty_mask : &none};
  return do_swap_out(p, items, out_n_moved);
}

int32_t swap_out_static(kv_pool_t* p, const int32_t* block_table, int32_t n_blocks, void* host_dst,
                        void* stream) {
  if (!p || n_blocks < 0 || (n_blocks > 0 && (!block_table || !host_dst))) return fail(KV_EINVAL, "bad argument");
  if (p->plan) return fail(KV_ENODEV, "a plan-only pool moves no bytes");
  if (n_blocks > KV_MAX_LAUNCH_BLOCKS || (int64_t)n_blocks * p->R > KV_STATIC_STAGING_BYTES)
    return fail(KV_EINVAL, "%d blocks (%lld bytes) exceed the static staging: at most %d blocks and %lld bytes per call",
                n_blocks, (long long)((int64_t)n_blocks * p->R), KV_MAX_LAUNCH_BLOCKS,
                (long long)KV_STATIC_STAGING_BYTES);
  if (!p->static_staging) return fail(KV_EHIP, "static staging has no address on this device");
  {
    std::lock_guard<std::mutex> g(p->mu);  // the duplicate stamps are shared with the other entry points
    ++p->epoch;
    for (int32_t i = 0; i < n_blocks; ++i) {
      const int64_t b = block_table[i];
      if (b < 0 || b >= p->N) return fail(KV_EINVAL, "block id %lld out of range [0,%lld)", (long long)b, (long long)p->N);
      if (p->stamp[(size_t)b] == p->epoch) return fail(KV_EINVAL, "block id %lld named twice", (long long)b);
      p->stamp[(size_t)b] = p->epoch;
    }
  }
  if (n_blocks == 0) return KV_OK;
  hipStream_t s = stream ? (hipStream_t)stream : p->s_pack;
  KvPackArgs a;  // on the stack: the block table travels in the kernel arguments
  a.pool = p->gpu;
  a.staging = p->static_staging;
  a.plane_stride = p->N * p->C;
  a.C = (uint32_t)p->C;
  a.P = (uint32_t)p->P;
  a.m = (uint32_t)n_blocks;
  a.tiles_per_chunk = a.n_tiles = a.xcd_blocks = 0;
  for (int32_t i = 0; i < n_blocks; ++i) a.table[i] = block_table[i];
  HIP_TRY(kv_launch_pack(false, a, p->unroll, p->variant, p->grid, s, nullptr, nullptr));
  HIP_TRY(hipMemcpyAsync(host_dst, p->static_staging, (size_t)n_blocks * (size_t)p->R, hipMemcpyDeviceToHost, s));
  if (!stream) HIP_TRY(hipStreamSynchronize(s));
  return KV_OK;
}

int32_t swap_in(kv_pool_t* p, int64_t req, const int32_t* new_block_table, int32_t n_blocks) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<InItem> items(1);
  items[0] = InItem{req, new_block_table, n_blocks, nullptr};
  return do_swap_in(p, items, nullptr);
}

int32_t swap_in_delta(kv_pool_t* p, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                      const uint8_t* resident_mask, int32_t* out_n_moved) {
  if (!p) return fail(KV_EINVAL, "null pool");
  if (n_blocks > 0 && !resident_mask) return fail(KV_EINVAL, "null resident mask");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<InItem> items(1);
  items[0] = InItem{req, new_block_table, n_blocks, resident_mask};
  return do_swap_in(p, items, out_n_moved);
}

int32_t swap_in_layerwise(kv_pool_t* p, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                          const uint8_t* resident_mask, int32_t layers_per_step, int32_t* out_n_moved) {
  if (!p) return fail(KV_EINVAL, "null pool");
  if (layers_per_step < 1 || layers_per_step > p->P / 2)
    return fail(KV_EINVAL, "layers_per_step %d outside [1, %d]", layers_per_step, p->P / 2);
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<InItem> items(1);
  items[0] = InItem{req, new_block_table, n_blocks, resident_mask};
  return do_swap_in(p, items, out_n_moved, 0, layers_per_step);
}

int32_t swap_out_direct(kv_pool_t* p, int64_t req, const int32_t* block_table, int32_t n_blocks,
                        int32_t per_block) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<OutItem> items(1);
  items[0] = OutItem{req, block_table, n_blocks, nullptr};
  return do_swap_out(p, items, nullptr, per_block ? 2 : 1);
}

int32_t swap_in_direct(kv_pool_t* p, int64_t req, const int32_t* new_block_table, int32_t n_blocks,
                       int32_t per_block) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<InItem> items(1);
  items[0] = InItem{req, new_block_table, n_blocks, nullptr};
  return do_swap_in(p, items, nullptr, per_block ? 2 : 1);
}

int32_t swap_out_batch(kv_pool_t* p, int32_t n_req, const int64_t* reqs, const int32_t* tables,
                       const int32_t* n_blocks) {
  if (!p || n_req < 0 || (n_req > 0 && (!reqs || !n_blocks))) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<OutItem> items((size_t)n_req);
  int64_t off = 0;
  for (int32_t i = 0; i < n_req; ++i) {
    if (n_blocks[i] < 0) return fail(KV_EINVAL, "negative table length");
    items[(size_t)i] = OutItem{reqs[i], tables + off, n_blocks[i], nullptr};
    off += n_blocks[i];
  }
  return do_swap_out(p, items, nullptr);
}

int32_t swap_in_batch(kv_pool_t* p, int32_t n_req, const int64_t* reqs, const int32_t* tables,
                      const int32_t* n_blocks) {
  if (!p || n_req < 0 || (n_req > 0 && (!reqs || !n_blocks))) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  std::vector<InItem> items((size_t)n_req);
  int64_t off = 0;
  for (int32_t i = 0; i < n_req; ++i) {
    if (n_blocks[i] < 0) return fail(KV_EINVAL, "negative table length");
    items[(size_t)i] = InItem{reqs[i], tables + off, n_blocks[i], nullptr};
    off += n_blocks[i];
  }
  return do_swap_in(p, items, nullptr);
}

static int32_t wait_event_unlocked(kv_pool* p, std::unique_lock<std::mutex>& lk, hipEvent_t ev) {
  if (p->plan || !ev) return KV_OK;
  lk.unlock();
  hipError_t e = hipEventSynchronize(ev);
  lk.lock();
  if (e != hipSuccess) return fail(KV_EHIP, "hipEventSynchronize: %s", hipGetErrorString(e));
  reap(p);
  return KV_OK;
}

int32_t kv_wait(kv_pool_t* p, int64_t req) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::unique_lock<std::mutex> lk(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end()) return fail(KV_ENOENT, "unknown request %lld", (long long)req);
  OpRef op = f->second.last;
  if (!op || op->all_done) return KV_OK;
  int32_t rc = wait_issued(p, op);
  if (rc) return rc;
  return wait_event_unlocked(p, lk, op->done);
}

int32_t kv_wait_packed(kv_pool_t* p, int64_t req) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::unique_lock<std::mutex> lk(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end()) return fail(KV_ENOENT, "unknown request %lld", (long long)req);
  OpRef op = f->second.last_out;
  if (!op || op->packed_done) return KV_OK;
  return wait_event_unlocked(p, lk, op->packed);
}

int32_t kv_query(kv_pool_t* p, int64_t req, int32_t* done) {
  if (!p || !done) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end()) return fail(KV_ENOENT, "unknown request %lld", (long long)req);
  reap(p);
  const OpRef& op = f->second.last;
  *done = (!op || op->all_done) ? 1 : 0;
  return KV_OK;
}

int32_t kv_stream_wait(kv_pool_t* p, int64_t req, void* stream) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end()) return fail(KV_ENOENT, "unknown request %lld", (long long)req);
  reap(p);
  const OpRef op = f->second.last;
  if (!op || op->all_done || p->plan) return KV_OK;
  int32_t rc = wait_issued(p, op);  // the event must have been recorded before a stream can wait for it
  if (rc) return rc;
  if (op->all_done) return KV_OK;
  HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, op->done, 0));
  return KV_OK;
}

// The event after which layer `layer` of req's last op is on the GPU: the step's own event
// for a layer-wise swap-in, the op's completion event otherwise.  Null = nothing to wait for.
static int32_t layer_event(kv_pool* p, int64_t req, int32_t layer, hipEvent_t* ev) {
  *ev = nullptr;
  if (layer < 0 || layer >= p->P / 2) return fail(KV_EINVAL, "layer %d outside [0, %d)", layer, p->P / 2);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end()) return fail(KV_ENOENT, "unknown request %lld", (long long)req);
  reap(p);
  const OpRef op = f->second.last;
  if (!op || op->all_done || p->plan) return KV_OK;
  int32_t rc = wait_issued(p, op);
  if (rc) return rc;
  if (op->all_done) return KV_OK;
  if (op->layer_step > 0 && !op->layer_ev.empty())
    *ev = op->layer_ev[(size_t)(layer / op->layer_step)];
  else
    *ev = op->done;
  return KV_OK;
}

int32_t kv_stream_wait_layer(kv_pool_t* p, int64_t req, int32_t layer, void* stream) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  hipEvent_t ev;
  int32_t rc = layer_event(p, req, layer, &ev);
  if (rc) return rc;
  if (ev) HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, ev, 0));
  return KV_OK;
}

int32_t kv_wait_layer(kv_pool_t* p, int64_t req, int32_t layer) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::unique_lock<std::mutex> lk(p->mu);
  hipEvent_t ev;
  int32_t rc = layer_event(p, req, layer, &ev);
  if (rc) return rc;
  if (!ev) return KV_OK;
  // not wait_event_unlocked: reaping here would be premature, the op's later steps still run
  lk.unlock();
  hipError_t e = hipEventSynchronize(ev);
  lk.lock();
  if (e != hipSuccess) return fail(KV_EHIP, "hipEventSynchronize: %s", hipGetErrorString(e));
  return KV_OK;
}

int32_t kv_wait_all(kv_pool_t* p) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::unique_lock<std::mutex> lk(p->mu);
  int32_t rc = wait_all_issued(p);
  if (rc) return rc;
  if (!p->plan) {
    // wait without the lock: other threads may keep enqueueing (their work is not waited for)
    const hipStream_t streams[4] = {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat};
    lk.unlock();
    hipError_t e = hipSuccess;
    for (hipStream_t s : streams)
      if (e == hipSuccess) e = hipStreamSynchronize(s);
    lk.lock();
    if (e != hipSuccess) return fail(KV_EHIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
  }
  reap(p);
  return KV_OK;
}

int32_t kv_host_len(kv_pool_t* p, int64_t req, int32_t* n_blocks, int32_t* n_extents) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  if (n_blocks) *n_blocks = f->second.img.n;
  if (n_extents) *n_extents = (int32_t)f->second.img.ext.size();
  return KV_OK;
}

int32_t kv_host_blocks(kv_pool_t* p, int64_t req, const void** arena_base, int64_t* record_index, int32_t n) {
  if (!p || (n > 0 && !record_index)) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  const Image& im = f->second.img;
  if (n != im.n) return fail(KV_EINVAL, "asked for %d blocks, host image has %d", n, im.n);
  if (arena_base) *arena_base = p->host;  // null in a plan-only pool: the records exist as bookkeeping only
  for (int32_t j = 0; j < n; ++j) record_index[j] = im.rec[(size_t)j];
  return KV_OK;
}

int32_t kv_host_read(kv_pool_t* p, int64_t req, int32_t first_block, int32_t n_blocks, void* dst) {
  if (!p || first_block < 0 || n_blocks < 0 || (n_blocks > 0 && !dst)) return fail(KV_EINVAL, "bad argument");
  std::unique_lock<std::mutex> lk(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  if ((int64_t)first_block + n_blocks > f->second.img.n)
    return fail(KV_EINVAL, "blocks [%d, %d) outside the host image of %d blocks", first_block,
                first_block + n_blocks, f->second.img.n);
  if (p->plan) return fail(KV_ENODEV, "a plan-only pool holds no bytes");
  OpRef op = f->second.last;
  if (op && !op->all_done) {
    int32_t rc = wait_issued(p, op);
    if (!rc) rc = wait_event_unlocked(p, lk, op->done);
    if (rc) return rc;
    f = p->reqs.find(req);  // the lock was dropped meanwhile
    if (f == p->reqs.end() || !f->second.has_image || (int64_t)first_block + n_blocks > f->second.img.n)
      return fail(KV_ENOENT, "request %lld lost its host copy during the wait", (long long)req);
  }
  // records of consecutive logical blocks are adjacent inside an extent: copy run by run
  const Image& im = f->second.img;
  char* out = (char*)dst;
  int32_t j = first_block;
  const int32_t end = first_block + n_blocks;
  while (j < end) {
    int32_t k = j;
    const int64_t r0 = im.rec[(size_t)j];
    if (r0 < 0) {
      while (k + 1 < end && im.rec[(size_t)k + 1] < 0) ++k;
      memset(out, 0, (size_t)(k - j + 1) * (size_t)p->R);
    } else {
      while (k + 1 < end && im.rec[(size_t)k + 1] == r0 + (k + 1 - j)) ++k;
      memcpy(out, p->host + r0 * p->R, (size_t)(k - j + 1) * (size_t)p->R);
    }
    out += (int64_t)(k - j + 1) * p->R;
    j = k + 1;
  }
  return KV_OK;
}

int32_t kv_host_view(kv_pool_t* p, int64_t req, const void** ptr, int64_t* bytes) {
  if (!p || !ptr || !bytes) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  if (p->plan) return fail(KV_ENODEV, "a plan-only pool holds no bytes");
  const Image& im = f->second.img;
  *bytes = (int64_t)im.n * p->R;
  *ptr = nullptr;
  if (im.n == 0) return KV_OK;
  const int64_t r0 = im.rec[0];
  if (r0 < 0) return KV_OK;
  for (int32_t j = 1; j < im.n; ++j)
    if (im.rec[(size_t)j] != r0 + j) return KV_OK;  // several extents, or records lost: use kv_host_read
  *ptr = p->host + r0 * p->R;
  return KV_OK;
}

int32_t kv_host_valid(kv_pool_t* p, int64_t req, uint8_t* out_mask, int32_t n) {
  if (!p || (n > 0 && !out_mask)) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  if (n != f->second.img.n) return fail(KV_EINVAL, "mask has %d entries, host image has %d blocks", n, f->second.img.n);
  if (n > 0) memcpy(out_mask, f->second.img.valid.data(), (size_t)n);
  return KV_OK;
}

int32_t kv_host_invalidate(kv_pool_t* p, int64_t req, const uint8_t* mask, int32_t n) {
  if (!p || (n > 0 && !mask)) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  if (n != f->second.img.n) return fail(KV_EINVAL, "mask has %d entries, host image has %d blocks", n, f->second.img.n);
  for (int32_t j = 0; j < n; ++j)
    if (mask[j]) f->second.img.valid[(size_t)j] = 0;
  return KV_OK;
}

int32_t kv_host_set_priority(kv_pool_t* p, int64_t req, int32_t priority) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  p->reqs[req].prio = priority;
  return KV_OK;
}

int32_t kv_host_release(kv_pool_t* p, int64_t req) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  int32_t rc = wait_all_issued(p);  // before the lookup: the lock is dropped during this wait
  if (rc) return rc;
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  rc = host_wait_op(p, f->second.last);
  if (rc) return rc;
  arena_give(p, f->second.img.ext);
  p->reqs.erase(f);
  return KV_OK;
}

int32_t kv_record_bytes(kv_pool_t* p, int64_t* out) {
  if (!p || !out) return fail(KV_EINVAL, "null argument");
  *out = p->R;
  return KV_OK;
}

int32_t kv_stats(kv_pool_t* p, kv_stats_t* out) {
  if (!p || !out) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  p->st.host_arena_bytes = p->arena_blocks * p->R;
  p->st.host_arena_used = (p->arena_blocks - p->arena.total()) * p->R;
  *out = p->st;
  return KV_OK;
}

int32_t kv_profile_read(kv_pool_t* p, kv_prof_record_t* out, int32_t cap, int32_t* out_n) {
  if (!p || !out_n) return fail(KV_EINVAL, "null argument");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->profile) return fail(KV_EINVAL, "pool was not created with KV_FLAG_PROFILE");
  int32_t rc = wait_all_issued(p);
  if (rc) return rc;
  for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat}) HIP_TRY(hipStreamSynchronize(s));
  *out_n = (int32_t)p->prof.size();
  for (int32_t i = 0; i < cap && i < *out_n; ++i) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, p->prof[(size_t)i].start, p->prof[(size_t)i].stop));
    out[i].kind = p->prof[(size_t)i].kind;
    out[i].reserved = 0;
    out[i].bytes = p->prof[(size_t)i].bytes;
    out[i].ms = ms;
    float t0 = 0.f;
    if (i > 0) HIP_TRY(hipEventElapsedTime(&t0, p->prof[0].start, p->prof[(size_t)i].start));
    out[i].start_ms = t0;
  }
  return KV_OK;
}

int32_t kv_profile_reset(kv_pool_t* p) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->profile) return KV_OK;
  int32_t rc = wait_all_issued(p);
  if (rc) return rc;
  for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat}) HIP_TRY(hipStreamSynchronize(s));
  for (auto& r : p->prof) {
    p->timing_pool.push_back(r.start);
    p->timing_pool.push_back(r.stop);
  }
  p->prof.clear();
  return KV_OK;
}

}  // extern "C"
