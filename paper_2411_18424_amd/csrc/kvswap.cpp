// Host side of the KV-swap library: pool object, reuse map, pinned host arena, staging
// rings, the event-ordered copy engine and the C ABI.
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
// Swap-out packs first and drains afterwards: all gathers of a call that fit the staging ring
// run back to back (the request's GPU blocks are reusable after about a millisecond), then
// the copies drain the ring; only a call larger than the ring interleaves the two.  Swap-in
// is pipelined piece by piece: the scatter of piece i runs under the copy of piece i+1.

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <chrono>
#include <deque>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/kvswap.h"
#include "kv_alloc.hpp"
#include "kv_kernels.h"

namespace {

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

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) return fail(KV_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

struct Op {
  uint64_t seq = 0;
  bool is_out = false;
  hipEvent_t packed = nullptr;  // swap-out only: recorded after the last gather
  hipEvent_t done = nullptr;    // recorded after the last copy (out) / scatter (in)
  bool packed_done = false, all_done = false;
  std::vector<hipEvent_t> aux;  // hand-off events of this op, recycled when it is done
};
using OpRef = std::shared_ptr<Op>;

// Host image of a request: its block records live in one or more extents of the pinned
// arena (Section 3.3: CPU space is reserved next to the copy for the next turn's increment;
// when that room is used up and the neighbour is taken, the image continues in a new extent
// instead of being moved).  rec[j] is the arena record that holds logical block j.
struct Extent {
  int64_t off = 0, cap = 0, used = 0;  // in block records
};

struct Image {
  std::vector<Extent> ext;
  int32_t n = 0;       // logical blocks
  int32_t mapped = 0;  // logical blocks [0, mapped) have a record; the rest lost theirs to eviction
  std::vector<uint8_t> valid;
  std::vector<int64_t> rec;  // -1 = no record
  int64_t room() const {
    int64_t r = 0;
    for (const Extent& e : ext) r += e.cap;
    return r;
  }
};

struct Req {
  bool has_image = false;
  Image img;
  OpRef last;      // last op of any kind
  OpRef last_out;  // last swap-out
  int32_t prio = 0;       // host copies of lower-priority requests are reclaimed first
  uint64_t last_use = 0;  // for least-recently-used order among equals
};

// Staging is a byte ring: a piece of a swap takes exactly the bytes it needs, so many small
// requests can be in flight at once and a large one wraps around.  Regions are handed out
// in ring order and retired in the same order.
struct Region {
  int64_t off = 0, len = 0;
  hipEvent_t freed = nullptr;  // recorded when the region's consumer has finished
  uint64_t op_seq = 0;
  bool recorded = false;
};

struct ByteRing {
  char* base = nullptr;
  int64_t cap = 0;
  int64_t head = 0;
  int64_t piece_blocks = 1;  // most blocks one piece carries
  std::deque<Region> live;
};

struct Move {
  int64_t host_off;  // byte offset in the arena of this logical block's record
  int32_t phys;
};

struct ProfRec {
  int32_t kind;
  int64_t bytes;
  hipEvent_t start, stop;
};

}  // namespace

struct kv_pool {
  kv_pool_config_t cfg{};
  bool plan = false, profile = false, order_compute = false, four_streams = false;
  int64_t N = 0, C = 0, R = 0;
  int32_t P = 0;
  char* gpu = nullptr;
  char* host = nullptr;      // pinned arena
  char* host_dev = nullptr;  // the arena as the device addresses it
  bool mapped_in = false;
  bool host_evict = false;
  uint64_t use_clock = 0;
  int mapped_grid = 64;
  int64_t arena_blocks = 0;
  bool own_staging = false;
  char* staging = nullptr;
  ByteRing ring_out, ring_in;
  hipStream_t s_pack = nullptr, s_d2h = nullptr, s_h2d = nullptr, s_scat = nullptr;
  hipStream_t compute = nullptr;
  hipEvent_t ev_compute = nullptr;
  int unroll = 0, grid = 0, variant = 0;
  int64_t launch_blocks = KV_MAX_LAUNCH_BLOCKS;  // most blocks one pack launch carries
  int64_t copy_chunk = 0;
  int64_t slack = 32;

  std::mutex mu;
  std::unordered_map<int64_t, Req> reqs;
  kv::RunSet arena;
  kv::BlockGroupAllocator alloc;
  kv::BlockGroupManager groups;
  std::vector<uint64_t> reader_seq, writer_seq;  // per physical block
  std::vector<uint32_t> stamp;                   // duplicate detection
  uint32_t epoch = 0;
  std::vector<uint32_t> free_stamp;
  uint32_t free_epoch = 0;

  std::deque<OpRef> ops_out, ops_in;
  uint64_t out_seq = 0, in_seq = 0;
  uint64_t pack_done_seq = 0, scat_done_seq = 0;
  std::vector<hipEvent_t> event_pool;   // timing disabled
  std::vector<hipEvent_t> timing_pool;  // timing enabled
  std::vector<ProfRec> prof;
  kv_stats_t st{};
};

namespace {

// ---------------------------------------------------------------- events
int32_t get_event(kv_pool* p, hipEvent_t* ev) {
  if (p->plan) {
    *ev = nullptr;
    return KV_OK;
  }
  if (!p->event_pool.empty()) {
    *ev = p->event_pool.back();
    p->event_pool.pop_back();
    return KV_OK;
  }
  HIP_TRY(hipEventCreateWithFlags(ev, hipEventDisableTiming));
  return KV_OK;
}

int32_t get_timing_event(kv_pool* p, hipEvent_t* ev) {
  if (!p->timing_pool.empty()) {
    *ev = p->timing_pool.back();
    p->timing_pool.pop_back();
    return KV_OK;
  }
  HIP_TRY(hipEventCreate(ev));
  return KV_OK;
}

void put_event(kv_pool* p, hipEvent_t ev) {
  if (ev) p->event_pool.push_back(ev);
}

// Polls completion of the oldest ops; recycles their events.  Ops of one direction finish
// in issue order (their kernels share one stream), so polling stops at the first unfinished.
void reap(kv_pool* p) {
  if (p->plan) {
    for (auto& o : p->ops_out) o->packed_done = o->all_done = true;
    for (auto& o : p->ops_in) o->all_done = true;
    p->pack_done_seq = p->out_seq;
    p->scat_done_seq = p->in_seq;
    p->ops_out.clear();
    p->ops_in.clear();
    p->ring_out.live.clear();
    p->ring_in.live.clear();
    p->alloc.reap(p->pack_done_seq);
    return;
  }
  for (auto& o : p->ops_out) {
    if (o->packed_done) continue;
    if (hipEventQuery(o->packed) != hipSuccess) break;
    o->packed_done = true;
    p->pack_done_seq = o->seq;
  }
  while (!p->ops_out.empty()) {
    Op& o = *p->ops_out.front();
    if (!o.packed_done || hipEventQuery(o.done) != hipSuccess) break;
    o.all_done = true;
    put_event(p, o.packed);
    put_event(p, o.done);
    o.packed = o.done = nullptr;
    for (hipEvent_t e : o.aux) put_event(p, e);
    o.aux.clear();
    p->ops_out.pop_front();
  }
  while (!p->ops_in.empty()) {
    Op& o = *p->ops_in.front();
    if (hipEventQuery(o.done) != hipSuccess) break;
    o.all_done = true;
    p->scat_done_seq = o.seq;
    put_event(p, o.done);
    o.done = nullptr;
    for (hipEvent_t e : o.aux) put_event(p, e);
    o.aux.clear();
    p->ops_in.pop_front();
  }
  for (ByteRing* r : {&p->ring_out, &p->ring_in}) {
    while (!r->live.empty()) {
      Region& f = r->live.front();
      if (!f.recorded || hipEventQuery(f.freed) != hipSuccess) break;
      put_event(p, f.freed);
      r->live.pop_front();
    }
  }
  p->alloc.reap(p->pack_done_seq);
}

Op* find_op(std::deque<OpRef>& dq, uint64_t seq) {
  if (dq.empty() || seq < dq.front()->seq) return nullptr;
  size_t i = (size_t)(seq - dq.front()->seq);
  return i < dq.size() ? dq[i].get() : nullptr;
}

// Host wait for one op (lock held by caller; short waits only on rare paths).
int32_t host_wait_op(kv_pool* p, const OpRef& op) {
  if (!op || op->all_done || p->plan) return KV_OK;
  if (op->done) HIP_TRY(hipEventSynchronize(op->done));
  reap(p);
  return KV_OK;
}

// ---------------------------------------------------------------- validation
int32_t check_table(kv_pool* p, const int32_t* t, int32_t n) {
  for (int32_t i = 0; i < n; ++i) {
    int64_t b = t[i];
    if (b < 0 || b >= p->N) return fail(KV_EINVAL, "block id %lld out of range [0,%lld)", (long long)b, (long long)p->N);
    if (p->stamp[(size_t)b] == p->epoch) return fail(KV_EINVAL, "block id %lld named twice", (long long)b);
    p->stamp[(size_t)b] = p->epoch;
  }
  return KV_OK;
}

// ---------------------------------------------------------------- host arena
// Takes room for n block records from the arena as few extents as it allows: one extent of
// n + slack if that fits, else exactly n, else the largest free runs until n is covered.
// New images are placed best-fit from the low end; a continuation extent of a grown image
// (spill) is taken from the high end of the largest free run, away from the tails of the
// packed images, so that it does not take the room the next image wants to grow into.
// Returns false (and takes nothing) when fewer than n records are free.
bool arena_take(kv_pool* p, int64_t n, std::vector<Extent>* out, bool spill) {
  if (n <= 0) return true;
  if (p->arena.total() < n) return false;
  int64_t off;
  if (spill && p->arena.take_top_of_largest(n + p->slack, &off)) {
    out->push_back({off, n + p->slack, 0});
    return true;
  }
  if (p->arena.take_best_fit(n + p->slack, &off)) {
    out->push_back({off, n + p->slack, 0});
    return true;
  }
  if (p->arena.take_best_fit(n, &off)) {
    out->push_back({off, n, 0});
    return true;
  }
  while (n > 0) {
    int64_t got = p->arena.take_from_largest(n, &off);
    out->push_back({off, got, 0});
    n -= got;
  }
  return true;
}

void arena_give(kv_pool* p, const std::vector<Extent>& ext) {
  for (const Extent& e : ext)
    if (e.cap > 0) p->arena.insert(e.off, e.cap);
}

// Lays logical blocks [from, to) onto the image's extents in order.
void image_map(Image& im, int32_t from, int32_t to) {
  im.rec.resize((size_t)to);
  size_t e = 0;
  for (int32_t j = from; j < to; ++j) {
    while (im.ext[e].used == im.ext[e].cap) ++e;
    im.rec[(size_t)j] = im.ext[e].off + im.ext[e].used++;
  }
}

// Gives the last k records of an image back to the arena: unused room first, then the records
// of its last logical blocks, which thereby lose their host copy (Section 3.3: the CPU copy is
// contaminated when its space is reclaimed for a higher-priority request).  Returns the number
// of logical blocks that lost their copy.
int64_t image_trim_tail(kv_pool* p, Image& im, int64_t k) {
  int64_t lost = 0;
  while (k > 0 && !im.ext.empty()) {
    Extent& e = im.ext.back();
    const int64_t cut = std::min(k, e.cap);
    const int64_t new_cap = e.cap - cut;
    if (e.used > new_cap) {
      const int64_t un = e.used - new_cap;
      for (int64_t i = 0; i < un; ++i) {
        const size_t j = (size_t)(--im.mapped);
        im.valid[j] = 0;
        im.rec[j] = -1;
      }
      lost += un;
      e.used = new_cap;
    }
    p->arena.insert(e.off + new_cap, cut);
    e.cap = new_cap;
    if (e.cap == 0) im.ext.pop_back();
    k -= cut;
  }
  return lost;
}

// KV_FLAG_HOST_EVICT: makes `need` records free by reclaiming the host copies of other
// requests - lowest priority first, least recently used first, never a request of higher
// priority than the caller's, never one whose last op is still in flight, never one named in
// `keep`.  All or nothing: returns false without touching anything if that is not enough.
bool arena_evict(kv_pool* p, int64_t need, int32_t prio, const std::vector<int64_t>& keep) {
  if (!p->host_evict) return false;
  struct Cand {
    int32_t prio;
    uint64_t last_use;
    int64_t req, room;
  };
  std::vector<Cand> cands;
  int64_t avail = p->arena.total();
  for (auto& kvp : p->reqs) {
    Req& q = kvp.second;
    if (!q.has_image || q.prio > prio) continue;
    if (q.last && !q.last->all_done) continue;
    if (std::find(keep.begin(), keep.end(), kvp.first) != keep.end()) continue;
    const int64_t room = q.img.room();
    if (room <= 0) continue;
    cands.push_back({q.prio, q.last_use, kvp.first, room});
    avail += room;
  }
  if (avail < need) return false;
  std::sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) {
    return a.prio != b.prio ? a.prio < b.prio : (a.last_use != b.last_use ? a.last_use < b.last_use : a.req < b.req);
  });
  for (const Cand& c : cands) {
    if (p->arena.total() >= need) break;
    Image& im = p->reqs[c.req].img;
    p->st.host_evicted_blocks += image_trim_tail(p, im, std::min(c.room, need - p->arena.total()));
  }
  return p->arena.total() >= need;
}

// ---------------------------------------------------------------- engine
int32_t stream_wait(kv_pool* p, hipStream_t s, hipEvent_t ev) {
  if (p->plan || !ev) return KV_OK;
  HIP_TRY(hipStreamWaitEvent(s, ev, 0));
  return KV_OK;
}

int32_t record(kv_pool* p, hipEvent_t ev, hipStream_t s) {
  if (p->plan || !ev) return KV_OK;
  HIP_TRY(hipEventRecord(ev, s));
  return KV_OK;
}

int32_t launch_pack(kv_pool* p, bool scatter, char* staging, const Move* mv, int64_t m) {
  hipStream_t s = scatter ? p->s_scat : p->s_pack;
  (scatter ? p->st.scatter_launches : p->st.gather_launches)++;
  if (p->plan) return KV_OK;
  KvPackArgs a;
  a.pool = p->gpu;
  a.staging = staging;
  a.plane_stride = p->N * p->C;
  a.C = (uint32_t)p->C;
  a.P = (uint32_t)p->P;
  a.m = (uint32_t)m;
  a.tiles_per_chunk = a.n_tiles = a.pad = 0;
  for (int64_t i = 0; i < m; ++i) a.table[i] = mv[i].phys;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (p->profile) {
    int32_t rc = get_timing_event(p, &e0);
    if (rc) return rc;
    rc = get_timing_event(p, &e1);
    if (rc) return rc;
    p->prof.push_back({scatter ? 1 : 0, m * p->R, e0, e1});
  }
  HIP_TRY(kv_launch_pack(scatter, a, p->unroll, p->variant, p->grid, s, e0, e1));
  return KV_OK;
}

// Copies of one ring slot: one copy per maximal run of moves whose host records are
// adjacent, each cut into pieces of at most copy_chunk bytes.
int32_t issue_copies(kv_pool* p, bool to_host, char* slot, const Move* mv, int64_t m) {
  hipStream_t s = to_host ? p->s_d2h : p->s_h2d;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (p->profile && !p->plan) {
    int32_t rc = get_timing_event(p, &e0);
    if (rc) return rc;
    rc = get_timing_event(p, &e1);
    if (rc) return rc;
    p->prof.push_back({to_host ? 2 : 3, m * p->R, e0, e1});
    HIP_TRY(hipEventRecord(e0, s));
  }
  int64_t i = 0;
  while (i < m) {
    int64_t j = i;
    while (j + 1 < m && mv[j + 1].host_off == mv[j].host_off + p->R) ++j;
    int64_t bytes = (j - i + 1) * p->R;
    char* h = p->host + mv[i].host_off;
    char* d = slot + i * p->R;
    for (int64_t o = 0; o < bytes; o += p->copy_chunk) {
      int64_t nb = std::min(p->copy_chunk, bytes - o);
      (to_host ? p->st.d2h_copies : p->st.h2d_copies)++;
      if (p->plan) continue;
      if (to_host)
        HIP_TRY(hipMemcpyAsync(h + o, d + o, (size_t)nb, hipMemcpyDeviceToHost, s));
      else
        HIP_TRY(hipMemcpyAsync(d + o, h + o, (size_t)nb, hipMemcpyHostToDevice, s));
    }
    i = j + 1;
  }
  if (e1) HIP_TRY(hipEventRecord(e1, s));
  return KV_OK;
}

int32_t order_after_compute(kv_pool* p, hipStream_t s) {
  if (!p->order_compute || p->plan) return KV_OK;
  HIP_TRY(hipEventRecord(p->ev_compute, p->compute));
  HIP_TRY(hipStreamWaitEvent(s, p->ev_compute, 0));
  return KV_OK;
}

// Claims `len` bytes at the ring head for op `op_seq`.  Every live region the claim
// overlaps (and every older one) must have been released by its consumer first: the
// producer stream is made to wait for it on the device.  `flush` is called before waiting
// on a region of the same op whose consumer work has not been issued yet.
template <class Flush>
int32_t ring_claim(kv_pool* p, ByteRing* r, int64_t len, uint64_t op_seq, hipStream_t producer,
                   Flush&& flush, Region** out) {
  int32_t rc;
  auto evict = [&](int64_t lo, int64_t hi) -> int32_t {
    int last = -1;
    for (int i = 0; i < (int)r->live.size(); ++i)
      if (r->live[(size_t)i].off < hi && lo < r->live[(size_t)i].off + r->live[(size_t)i].len) last = i;
    for (int i = 0; i <= last; ++i) {
      if (!r->live.front().recorded) {
        if (r->live.front().op_seq != op_seq) return fail(KV_EBUSY, "staging region of another call is still open");
        if ((rc = flush())) return rc;
      }
      Region f = r->live.front();
      r->live.pop_front();
      if ((rc = stream_wait(p, producer, f.freed))) return rc;
      put_event(p, f.freed);
    }
    return KV_OK;
  };
  if (r->head + len > r->cap) {  // the tail is too short: skip it and start over at 0
    if ((rc = evict(r->head, r->cap))) return rc;
    r->head = 0;
  }
  if ((rc = evict(r->head, r->head + len))) return rc;
  Region g;
  g.off = r->head;
  g.len = len;
  g.op_seq = op_seq;
  if ((rc = get_event(p, &g.freed))) return rc;
  r->head += len;
  r->live.push_back(g);
  *out = &r->live.back();
  return KV_OK;
}

// Swap-out of a move list: gather pieces into the staging ring, then drain them to the host.
// pre: events the first gather must wait for.
int32_t enqueue_out(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                    const OpRef& op) {
  int32_t rc;
  if ((rc = order_after_compute(p, p->s_pack))) return rc;
  for (hipEvent_t e : pre)
    if ((rc = stream_wait(p, p->s_pack, e))) return rc;
  ByteRing& r = p->ring_out;
  const int64_t m = (int64_t)mv.size();
  struct Pending {
    int64_t first, count, off;
  };
  std::vector<Pending> pending;  // gathered, copies not issued yet
  auto flush = [&]() -> int32_t {
    if (pending.empty()) return KV_OK;
    int32_t rc2;
    hipEvent_t ready;
    if ((rc2 = get_event(p, &ready))) return rc2;
    if (ready) op->aux.push_back(ready);
    if ((rc2 = record(p, ready, p->s_pack))) return rc2;
    if ((rc2 = stream_wait(p, p->s_d2h, ready))) return rc2;
    for (const Pending& q : pending) {
      if ((rc2 = issue_copies(p, true, r.base + q.off, &mv[(size_t)q.first], q.count))) return rc2;
      for (Region& g : r.live)
        if (g.off == q.off && g.op_seq == op->seq && !g.recorded) {
          if ((rc2 = record(p, g.freed, p->s_d2h))) return rc2;
          g.recorded = true;
        }
    }
    pending.clear();
    return KV_OK;
  };
  for (int64_t i = 0; i < m; i += r.piece_blocks) {
    const int64_t mp = std::min(r.piece_blocks, m - i);
    Region* g;
    if ((rc = ring_claim(p, &r, mp * p->R, op->seq, p->s_pack, flush, &g))) return rc;
    const int64_t off = g->off;
    for (int64_t k = 0; k < mp; k += p->launch_blocks) {
      int64_t ml = std::min<int64_t>(p->launch_blocks, mp - k);
      if ((rc = launch_pack(p, false, r.base + off + k * p->R, &mv[(size_t)(i + k)], ml))) return rc;
    }
    pending.push_back({i, mp, off});
  }
  if ((rc = record(p, op->packed, p->s_pack))) return rc;
  if ((rc = flush())) return rc;
  if (m == 0 && (rc = stream_wait(p, p->s_d2h, op->packed))) return rc;
  if ((rc = record(p, op->done, p->s_d2h))) return rc;
  p->st.bytes_out += m * p->R;
  p->st.blocks_out += m;
  return KV_OK;
}

// Swap-in of a move list: copy host records into ring pieces, scatter each piece.
// pre_copy: events the first host-to-device copy waits for (the image's last writer);
// pre_scat: events the first scatter waits for (gathers still reading the target blocks).
int32_t enqueue_in(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre_copy,
                   const std::vector<hipEvent_t>& pre_scat, const OpRef& op) {
  int32_t rc;
  for (hipEvent_t e : pre_copy)
    if ((rc = stream_wait(p, p->s_h2d, e))) return rc;
  if ((rc = order_after_compute(p, p->s_scat))) return rc;
  for (hipEvent_t e : pre_scat)
    if ((rc = stream_wait(p, p->s_scat, e))) return rc;
  ByteRing& r = p->ring_in;
  const int64_t m = (int64_t)mv.size();
  auto no_flush = []() -> int32_t { return KV_OK; };  // every region is closed before the next claim
  for (int64_t i = 0; i < m; i += r.piece_blocks) {
    const int64_t mp = std::min(r.piece_blocks, m - i);
    Region* g;
    if ((rc = ring_claim(p, &r, mp * p->R, op->seq, p->s_h2d, no_flush, &g))) return rc;
    char* sb = r.base + g->off;
    if ((rc = issue_copies(p, false, sb, &mv[(size_t)i], mp))) return rc;
    hipEvent_t ready;
    if ((rc = get_event(p, &ready))) return rc;
    if (ready) op->aux.push_back(ready);
    if ((rc = record(p, ready, p->s_h2d))) return rc;
    if ((rc = stream_wait(p, p->s_scat, ready))) return rc;
    for (int64_t k = 0; k < mp; k += p->launch_blocks) {
      int64_t ml = std::min<int64_t>(p->launch_blocks, mp - k);
      if ((rc = launch_pack(p, true, sb + k * p->R, &mv[(size_t)(i + k)], ml))) return rc;
    }
    if ((rc = record(p, g->freed, p->s_scat))) return rc;
    g->recorded = true;
  }
  if (m == 0) {
    // nothing moved: completion still follows the image's last writer
    for (hipEvent_t e : pre_copy)
      if ((rc = stream_wait(p, p->s_scat, e))) return rc;
  }
  if ((rc = record(p, op->done, p->s_scat))) return rc;
  p->st.bytes_in += m * p->R;
  p->st.blocks_in += m;
  return KV_OK;
}

// Comparison path: the paper's own transfer scheme (Section 3.1, one copy per contiguous
// block group) on this pool layout, without a pack kernel.  A run of r physically adjacent
// blocks is r*C contiguous bytes in each of the P planes of the pool and r records R bytes
// apart in the host image, so it takes one 2-D copy per (run, plane); per_block cuts every
// run into single blocks (one copy per block and plane, the per-block baseline of Section
// 2.2).  Everything runs on the copy stream; the blocks stay busy until the transfer ends.
int32_t enqueue_direct(kv_pool* p, bool to_host, const std::vector<Move>& mv,
                       const std::vector<hipEvent_t>& pre, const OpRef& op, bool per_block) {
  int32_t rc;
  hipStream_t s = to_host ? p->s_d2h : p->s_h2d;
  if ((rc = order_after_compute(p, s))) return rc;
  for (hipEvent_t e : pre)
    if ((rc = stream_wait(p, s, e))) return rc;
  const int64_t m = (int64_t)mv.size();
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (p->profile && !p->plan && m > 0) {
    if ((rc = get_timing_event(p, &e0))) return rc;
    if ((rc = get_timing_event(p, &e1))) return rc;
    p->prof.push_back({to_host ? 2 : 3, m * p->R, e0, e1});
    HIP_TRY(hipEventRecord(e0, s));
  }
  int64_t i = 0;
  while (i < m) {
    int64_t j = i;
    if (!per_block)
      while (j + 1 < m && mv[(size_t)j + 1].phys == mv[(size_t)j].phys + 1 &&
             mv[(size_t)j + 1].host_off == mv[(size_t)j].host_off + p->R)
        ++j;
    const int64_t r = j - i + 1;
    for (int32_t pl = 0; pl < p->P; ++pl) {
      char* h = p->host + mv[(size_t)i].host_off + (int64_t)pl * p->C;
      char* d = p->gpu + ((int64_t)pl * p->N + mv[(size_t)i].phys) * p->C;
      (to_host ? p->st.d2h_copies : p->st.h2d_copies)++;
      if (p->plan) continue;
      if (to_host)
        HIP_TRY(hipMemcpy2DAsync(h, (size_t)p->R, d, (size_t)p->C, (size_t)p->C, (size_t)r,
                                 hipMemcpyDeviceToHost, s));
      else
        HIP_TRY(hipMemcpy2DAsync(d, (size_t)p->C, h, (size_t)p->R, (size_t)p->C, (size_t)r,
                                 hipMemcpyHostToDevice, s));
    }
    i = j + 1;
  }
  if (e1) HIP_TRY(hipEventRecord(e1, s));
  if (to_host && (rc = record(p, op->packed, s))) return rc;
  if ((rc = record(p, op->done, s))) return rc;
  (to_host ? p->st.bytes_out : p->st.bytes_in) += m * p->R;
  (to_host ? p->st.blocks_out : p->st.blocks_in) += m;
  return KV_OK;
}

// Swap-in straight from the pinned image (KV_FLAG_MAPPED_SWAP_IN): one persistent kernel per
// 440 blocks reads the host records over the link and writes the pool; no staging, no copy
// engine, no per-run copies - fragmented images and partial swap-ins cost the same as
// contiguous ones.
int32_t enqueue_in_mapped(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                          const OpRef& op) {
  int32_t rc;
  hipStream_t s = p->s_scat;
  if ((rc = order_after_compute(p, s))) return rc;
  for (hipEvent_t e : pre)
    if ((rc = stream_wait(p, s, e))) return rc;
  const int64_t m = (int64_t)mv.size();
  for (int64_t i = 0; i < m; i += KV_MAX_MAPPED_BLOCKS) {
    const int64_t ml = std::min<int64_t>(KV_MAX_MAPPED_BLOCKS, m - i);
    p->st.scatter_launches++;
    if (p->plan) continue;
    KvMappedArgs a;
    a.pool = p->gpu;
    a.host = p->host_dev;
    a.plane_stride = p->N * p->C;
    a.R = p->R;
    a.C = (uint32_t)p->C;
    a.P = (uint32_t)p->P;
    a.m = (uint32_t)ml;
    a.tiles_per_chunk = a.n_tiles = a.pad = 0;
    for (int64_t k = 0; k < ml; ++k) {
      a.phys[k] = mv[(size_t)(i + k)].phys;
      a.rec[k] = (uint32_t)(mv[(size_t)(i + k)].host_off / p->R);
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (p->profile) {
      if ((rc = get_timing_event(p, &e0))) return rc;
      if ((rc = get_timing_event(p, &e1))) return rc;
      p->prof.push_back({4, ml * p->R, e0, e1});
    }
    HIP_TRY(kv_launch_mapped_scatter(a, p->mapped_grid, s, e0, e1));
  }
  if ((rc = record(p, op->done, s))) return rc;
  p->st.bytes_in += m * p->R;
  p->st.blocks_in += m;
  return KV_OK;
}

int32_t new_op(kv_pool* p, bool is_out, OpRef* out) {
  auto op = std::make_shared<Op>();
  op->is_out = is_out;
  int32_t rc;
  if (is_out) {
    if ((rc = get_event(p, &op->packed))) return rc;
  }
  if ((rc = get_event(p, &op->done))) return rc;
  op->seq = is_out ? ++p->out_seq : ++p->in_seq;
  (is_out ? p->ops_out : p->ops_in).push_back(op);
  *out = op;
  return KV_OK;
}

// One request of a (possibly batched) swap-out, after validation.
struct OutItem {
  int64_t req;
  const int32_t* table;
  int32_t n;
  const uint8_t* dirty;  // null = full swap-out
  // planning results
  bool fresh = false;             // image is (re)built on new extents; the old ones are given back
  int64_t extend_last_by = 0;     // the last extent grows in place by this many records
  std::vector<Extent> new_ext;    // extents taken from the arena for this call
};

int32_t do_swap_out(kv_pool* p, std::vector<OutItem>& items, int32_t* out_n_moved, int direct = 0) {
  reap(p);
  int32_t rc;
  // 1. validate tables (ids unique across the whole call) and shapes
  ++p->epoch;
  for (size_t a = 0; a < items.size(); ++a) {
    OutItem& it = items[a];
    if (it.n < 0 || (it.n > 0 && !it.table)) return fail(KV_EINVAL, "bad table");
    for (size_t b = 0; b < a; ++b)
      if (items[b].req == it.req) return fail(KV_EINVAL, "request %lld named twice", (long long)it.req);
    if ((rc = check_table(p, it.table, it.n))) return rc;
    auto f = p->reqs.find(it.req);
    if (it.dirty && f != p->reqs.end() && f->second.has_image && it.n < f->second.img.n)
      return fail(KV_EINVAL, "table (%d blocks) shorter than the host image (%d)", it.n, f->second.img.n);
  }
  // 2. plan host space without touching existing images; undo on failure
  auto undo = [&](size_t upto) {
    for (size_t a = 0; a < upto; ++a) {
      arena_give(p, items[a].new_ext);
      if (items[a].extend_last_by > 0) {
        const Extent& last = p->reqs[items[a].req].img.ext.back();
        p->arena.insert(last.off + last.cap, items[a].extend_last_by);
      }
    }
  };
  for (size_t a = 0; a < items.size(); ++a) {
    OutItem& it = items[a];
    auto f = p->reqs.find(it.req);
    const bool has = f != p->reqs.end() && f->second.has_image;
    int64_t need = it.n;
    if (has) {
      Image& im = f->second.img;
      if (it.n <= im.room()) continue;  // fits the room already reserved
      if (it.dirty) {
        // append: first try to grow the last extent where it stands
        need = it.n - im.room();
        if (!im.ext.empty()) {
          const Extent& last = im.ext.back();
          if (p->arena.take_exact(last.off + last.cap, need + p->slack)) {
            it.extend_last_by = need + p->slack;
            continue;
          }
          if (p->arena.take_exact(last.off + last.cap, need)) {
            it.extend_last_by = need;
            continue;
          }
        }
      } else {
        it.fresh = true;  // a full swap-out that outgrew the old image starts over
      }
    } else {
      it.fresh = true;
    }
    bool got = arena_take(p, need, &it.new_ext, !it.fresh);
    if (!got) {
      // reclaim host copies of lower-priority requests (not those of this very call)
      std::vector<int64_t> keep;
      for (const OutItem& o : items) keep.push_back(o.req);
      auto fq = p->reqs.find(it.req);
      got = arena_evict(p, need, fq != p->reqs.end() ? fq->second.prio : 0, keep) &&
            arena_take(p, need, &it.new_ext, !it.fresh);
    }
    if (!got) {
      undo(a);
      return fail(KV_ENOMEM_HOST, "host arena full: need %lld block records, %lld free (largest run %lld)",
                  (long long)need, (long long)p->arena.total(), (long long)p->arena.largest());
    }
  }
  // 3. commit: images, reuse map, move list
  std::vector<Move> mv;
  std::vector<hipEvent_t> pre;
  uint64_t max_writer = 0;
  OpRef op;
  if ((rc = new_op(p, true, &op))) {
    undo(items.size());
    return rc;
  }
  int64_t total_moved = 0;
  for (OutItem& it : items) {
    Req& q = p->reqs[it.req];
    Image& im = q.img;
    if (it.fresh) {
      if (q.has_image) {
        // the old extents may still be read or written by an unfinished op of this request
        if ((rc = host_wait_op(p, q.last))) return rc;
        arena_give(p, im.ext);
      }
      im.ext = it.new_ext;
      im.n = im.mapped = 0;
      im.valid.clear();
      im.rec.clear();
      q.has_image = true;
    } else {
      if (it.extend_last_by > 0) im.ext.back().cap += it.extend_last_by;
      if (!it.new_ext.empty()) {
        im.ext.insert(im.ext.end(), it.new_ext.begin(), it.new_ext.end());
        p->st.host_new_extents += (int64_t)it.new_ext.size();
      }
    }
    if (!it.dirty) {  // full swap-out: the earlier copy is discarded, blocks are laid out anew
      for (Extent& e : im.ext) e.used = 0;
      im.n = it.n;
      im.valid.assign((size_t)it.n, 0);
      image_map(im, 0, it.n);
    } else {
      if (it.n > im.n) {
        im.valid.resize((size_t)it.n, 0);
        im.n = it.n;
      }
      if (im.mapped < im.n) image_map(im, im.mapped, im.n);  // new blocks, and blocks that lost their record
    }
    im.mapped = im.n;
    q.last_use = ++p->use_clock;
    int32_t moved = 0;
    for (int32_t j = 0; j < it.n; ++j) {
      if (it.dirty && !it.dirty[j] && q.img.valid[(size_t)j]) continue;
      q.img.valid[(size_t)j] = 1;
      int32_t b = it.table[j];
      mv.push_back({q.img.rec[(size_t)j] * p->R, b});
      p->reader_seq[(size_t)b] = op->seq;
      max_writer = std::max(max_writer, p->writer_seq[(size_t)b]);
      ++moved;
    }
    total_moved += moved;
    // ops of one request are serialised: this gather follows the request's last op
    if (q.last && !q.last->all_done && q.last->done) pre.push_back(q.last->done);
    q.last = op;
    q.last_out = op;
  }
  if (max_writer > p->scat_done_seq) {  // a scatter into these blocks is still in flight
    if (Op* w = find_op(p->ops_in, max_writer)) {
      if (w->done) {
        pre.push_back(w->done);
        p->st.conflict_waits++;
      }
    }
  }
  if (out_n_moved) *out_n_moved = (int32_t)total_moved;
  if (direct) return enqueue_direct(p, true, mv, pre, op, direct == 2);
  return enqueue_out(p, mv, pre, op);
}

struct InItem {
  int64_t req;
  const int32_t* table;
  int32_t n;
  const uint8_t* resident;  // null = move everything
};

int32_t do_swap_in(kv_pool* p, std::vector<InItem>& items, int32_t* out_n_moved, int direct = 0) {
  reap(p);
  int32_t rc;
  ++p->epoch;
  for (size_t a = 0; a < items.size(); ++a) {
    InItem& it = items[a];
    if (it.n < 0 || (it.n > 0 && !it.table)) return fail(KV_EINVAL, "bad table");
    for (size_t b = 0; b < a; ++b)
      if (items[b].req == it.req) return fail(KV_EINVAL, "request %lld named twice", (long long)it.req);
    auto f = p->reqs.find(it.req);
    if (f == p->reqs.end() || !f->second.has_image)
      return fail(KV_ENOENT, "request %lld has no host copy", (long long)it.req);
    if (f->second.img.n != it.n)
      return fail(KV_EINVAL, "table has %d blocks, host image has %d", it.n, f->second.img.n);
    if ((rc = check_table(p, it.table, it.n))) return rc;
    for (int32_t j = 0; j < it.n; ++j) {
      if (it.resident && it.resident[j]) continue;
      if (!f->second.img.valid[(size_t)j])
        return fail(KV_ENOENT, "request %lld: logical block %d has no valid host copy", (long long)it.req, j);
    }
  }
  OpRef op;
  if ((rc = new_op(p, false, &op))) return rc;
  std::vector<Move> mv;
  std::vector<hipEvent_t> pre_copy, pre_scat;
  uint64_t max_reader = 0;
  for (InItem& it : items) {
    Req& q = p->reqs[it.req];
    for (int32_t j = 0; j < it.n; ++j) {
      if (it.resident && it.resident[j]) continue;
      int32_t b = it.table[j];
      mv.push_back({q.img.rec[(size_t)j] * p->R, b});
      p->writer_seq[(size_t)b] = op->seq;
      max_reader = std::max(max_reader, p->reader_seq[(size_t)b]);
    }
    if (q.last && !q.last->all_done && q.last->done) pre_copy.push_back(q.last->done);
    q.last = op;
    q.last_use = ++p->use_clock;
  }
  if (max_reader > p->pack_done_seq) {  // a gather still reads blocks we are about to overwrite
    if (Op* r = find_op(p->ops_out, max_reader)) {
      if (r->packed && !r->packed_done) {
        pre_scat.push_back(r->packed);
        p->st.conflict_waits++;
      }
    }
  }
  if (out_n_moved) *out_n_moved = (int32_t)mv.size();
  if (direct) {
    pre_copy.insert(pre_copy.end(), pre_scat.begin(), pre_scat.end());
    return enqueue_direct(p, false, mv, pre_copy, op, direct == 2);
  }
  if (p->mapped_in) {
    pre_copy.insert(pre_copy.end(), pre_scat.begin(), pre_scat.end());
    return enqueue_in_mapped(p, mv, pre_copy, op);
  }
  return enqueue_in(p, mv, pre_copy, pre_scat, op);
}

void destroy_pool(kv_pool* p) {
  if (!p->plan) {
    (void)hipDeviceSynchronize();
    for (ByteRing* r : {&p->ring_out, &p->ring_in})
      for (Region& g : r->live)
        if (g.freed) (void)hipEventDestroy(g.freed);
    for (auto* dq : {&p->ops_out, &p->ops_in})
      for (auto& o : *dq) {
        if (o->packed) (void)hipEventDestroy(o->packed);
        if (o->done) (void)hipEventDestroy(o->done);
        for (hipEvent_t e : o->aux) (void)hipEventDestroy(e);
      }
    for (hipEvent_t e : p->event_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->timing_pool) (void)hipEventDestroy(e);
    for (auto& r : p->prof) {
      (void)hipEventDestroy(r.start);
      (void)hipEventDestroy(r.stop);
    }
    if (p->ev_compute) (void)hipEventDestroy(p->ev_compute);
    if (!p->four_streams) p->s_d2h = p->s_scat = nullptr;  // aliases of the other two
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
  p->copy_chunk = cfg->copy_chunk_bytes > 0 ? cfg->copy_chunk_bytes : (64ll << 20);
  p->grid = cfg->gather_grid;
  p->unroll = cfg->tile_unroll;  // 0 = pick from the chunk size
  p->variant = cfg->pack_variant;
  p->mapped_in = (cfg->flags & KV_FLAG_MAPPED_SWAP_IN) != 0;
  p->host_evict = (cfg->flags & KV_FLAG_HOST_EVICT) != 0;
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
  p->ring_out.piece_blocks = piece_blocks(out_cap, p->launch_blocks * p->R);
  p->ring_in.cap = in_cap;
  p->ring_in.piece_blocks = piece_blocks(in_cap, 256ll << 20);
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
    }
    TRY_OR_BAIL(hipEventCreateWithFlags(&p->ev_compute, hipEventDisableTiming));
    if (p->arena_blocks > 0) {
      hipError_t e = hipHostMalloc((void**)&p->host, (size_t)(p->arena_blocks * p->R), hipHostMallocDefault);
      if (e != hipSuccess) return bail(fail(KV_ENOMEM_HOST, "hipHostMalloc(%lld): %s", (long long)(p->arena_blocks * p->R), hipGetErrorString(e)));
      TRY_OR_BAIL(hipHostGetDevicePointer((void**)&p->host_dev, p->host, 0));
    }
    if (cfg->staging_base) {
      p->staging = (char*)cfg->staging_base;
    } else {
      hipError_t e = hipMalloc((void**)&p->staging, (size_t)(out_cap + in_cap));
      if (e != hipSuccess) return bail(fail(KV_ENOMEM_GPU, "hipMalloc(staging %lld): %s", (long long)(out_cap + in_cap), hipGetErrorString(e)));
      p->own_staging = true;
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

int32_t alloc_block_group(kv_pool_t* p, int64_t req, int32_t n_blocks, int32_t min_run,
                          int32_t* out_blocks, int32_t* out_n_runs) {
  (void)req;
  if (!p || n_blocks < 0 || (n_blocks > 0 && !out_blocks)) return fail(KV_EINVAL, "bad argument");
  std::lock_guard<std::mutex> g(p->mu);
  reap(p);
  if (p->alloc.n_free() < n_blocks) {
    // blocks parked behind an unfinished gather may cover the shortfall: wait for exactly
    // the gather that releases enough of them (fine-grained conflict synchronisation)
    if (p->alloc.n_free() + p->alloc.n_draining() < n_blocks)
      return fail(KV_ENOMEM_GPU, "need %d blocks, %lld free", n_blocks,
                  (long long)(p->alloc.n_free() + p->alloc.n_draining()));
    uint64_t seq = p->alloc.seq_to_release(n_blocks - p->alloc.n_free());
    Op* o = find_op(p->ops_out, seq);
    if (o && o->packed && !o->packed_done && !p->plan) {
      HIP_TRY(hipEventSynchronize(o->packed));
      p->st.conflict_waits++;
    }
    reap(p);
    if (p->alloc.n_free() < n_blocks) return fail(KV_ENOMEM_GPU, "need %d blocks, %lld free", n_blocks, (long long)p->alloc.n_free());
  }
  std::vector<int32_t> ids;
  ids.reserve((size_t)n_blocks);
  int32_t runs = p->alloc.alloc(n_blocks, min_run, &ids);
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
  p->alloc.free_ids(blocks, n_blocks, p->reader_seq, p->pack_done_seq);
  return KV_OK;
}

// Waits (fine-grained) for gathers that still read parked blocks until `need` blocks are free.
static int32_t make_free(kv_pool* p, int64_t need) {
  reap(p);
  while (p->alloc.n_free() < need && p->alloc.n_draining() > 0) {
    uint64_t seq = p->alloc.seq_to_release(std::min(need - p->alloc.n_free(), p->alloc.n_draining()));
    Op* o = find_op(p->ops_out, seq);
    if (o && o->packed && !o->packed_done && !p->plan) {
      HIP_TRY(hipEventSynchronize(o->packed));
      p->st.conflict_waits++;
    }
    int64_t before = p->alloc.n_draining();
    reap(p);
    if (p->alloc.n_draining() == before) break;
  }
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
  p->alloc.free_ids(ids.data(), (int32_t)ids.size(), p->reader_seq, p->pack_done_seq);
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
  const OpRef& op = f->second.last;
  if (!op || op->all_done || p->plan) return KV_OK;
  HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, op->done, 0));
  return KV_OK;
}

int32_t kv_wait_all(kv_pool_t* p) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->plan) {
    for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat}) HIP_TRY(hipStreamSynchronize(s));
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
  if (p->plan) return fail(KV_ENODEV, "plan-only pool holds no bytes");
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  const Image& im = f->second.img;
  if (n != im.n) return fail(KV_EINVAL, "asked for %d blocks, host image has %d", n, im.n);
  if (arena_base) *arena_base = p->host;
  for (int32_t j = 0; j < n; ++j) record_index[j] = im.rec[(size_t)j];
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
  auto f = p->reqs.find(req);
  if (f == p->reqs.end() || !f->second.has_image) return fail(KV_ENOENT, "request %lld has no host copy", (long long)req);
  int32_t rc = host_wait_op(p, f->second.last);
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
  for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat}) HIP_TRY(hipStreamSynchronize(s));
  *out_n = (int32_t)p->prof.size();
  for (int32_t i = 0; i < cap && i < *out_n; ++i) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, p->prof[(size_t)i].start, p->prof[(size_t)i].stop));
    out[i].kind = p->prof[(size_t)i].kind;
    out[i].reserved = 0;
    out[i].bytes = p->prof[(size_t)i].bytes;
    out[i].ms = ms;
  }
  return KV_OK;
}

int32_t kv_profile_reset(kv_pool_t* p) {
  if (!p) return fail(KV_EINVAL, "null pool");
  std::lock_guard<std::mutex> g(p->mu);
  if (!p->profile) return KV_OK;
  for (hipStream_t s : {p->s_pack, p->s_d2h, p->s_h2d, p->s_scat}) HIP_TRY(hipStreamSynchronize(s));
  for (auto& r : p->prof) {
    p->timing_pool.push_back(r.start);
    p->timing_pool.push_back(r.stop);
  }
  p->prof.clear();
  return KV_OK;
}

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
  PROBE_TRY(hipMemcpyAsync(d0, h0, (size_t)bytes, hipMemcpyHostToDevice, s0));  // warm-up, fills d0
  if (direction == 2) PROBE_TRY(hipMemcpyAsync(d1, h1, (size_t)bytes, hipMemcpyHostToDevice, s1));
  PROBE_TRY(hipStreamSynchronize(s0));
  PROBE_TRY(hipStreamSynchronize(s1));
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
