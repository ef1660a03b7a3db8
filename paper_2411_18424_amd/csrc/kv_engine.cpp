// Copy engine of the KV-swap library: event pool, completion polling, staging byte rings,
// pack-kernel launches, host-link copies and their ordering (FastSwitch, arXiv 2411.18424,
// Section 3.2: asynchronous swapping on side streams, progress recorded with pooled events,
// conflicts resolved by waiting for exactly the transfer concerned).
//
// Swap-out packs first and drains afterwards where gathers and copies share a stream (the
// default): all gathers of a call that fit the staging ring run back to back (the request's
// GPU blocks are reusable after about a millisecond), then the copies drain the ring; only a
// call larger than the ring interleaves the two.  With KV_FLAG_FOUR_STREAMS the copies of a
// piece are issued right behind its gather and the later gathers run under them.  Swap-in is
// pipelined piece by piece.

#include <algorithm>

#include "kv_pool.hpp"

namespace kvi {

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
// in issue order (their completion events are recorded on one stream per direction), so polling
// stops at the first unfinished one - and at an op that is still being enqueued (its events
// have not been recorded yet, and an unrecorded event reads as complete).
void reap(kv_pool* p) {
  if (p->plan) {  // nothing runs: whatever has been enqueued is done
    while (!p->ops_out.empty() && p->ops_out.front()->issued) {
      Op& o = *p->ops_out.front();
      o.packed_done = o.all_done = true;
      p->pack_done_seq = o.seq;
      p->ops_out.pop_front();
    }
    while (!p->ops_in.empty() && p->ops_in.front()->issued) {
      Op& o = *p->ops_in.front();
      o.all_done = true;
      p->scat_done_seq = o.seq;
      p->ops_in.pop_front();
    }
    p->ring_out.live.clear();
    p->ring_in.live.clear();
    p->alloc.reap(p->pack_done_seq, p->scat_done_seq);
    return;
  }
  for (auto& o : p->ops_out) {
    if (o->packed_done) continue;
    if (!o->packed_recorded || p->event_query(o->packed) != hipSuccess) break;
    o->packed_done = true;
    p->pack_done_seq = o->seq;
  }
  while (!p->ops_out.empty()) {
    Op& o = *p->ops_out.front();
    if (!o.issued || !o.packed_done || p->event_query(o.done) != hipSuccess) break;
    o.all_done = true;
    put_event(p, o.packed);
    put_event(p, o.done);
    o.packed = o.done = nullptr;
    for (hipEvent_t e : o.aux) put_event(p, e);
    o.aux.clear();
    for (hipEvent_t e : o.timed) p->timing_pool.push_back(e);
    o.timed.clear();
    p->ops_out.pop_front();
  }
  while (!p->ops_in.empty()) {
    Op& o = *p->ops_in.front();
    if (!o.issued || p->event_query(o.done) != hipSuccess) break;
    o.all_done = true;
    p->scat_done_seq = o.seq;
    put_event(p, o.done);
    o.done = nullptr;
    for (hipEvent_t e : o.aux) put_event(p, e);
    o.aux.clear();
    for (hipEvent_t e : o.layer_ev) put_event(p, e);
    o.layer_ev.clear();
    for (hipEvent_t e : o.timed) p->timing_pool.push_back(e);
    o.timed.clear();
    p->ops_in.pop_front();
  }
  for (ByteRing* r : {&p->ring_out, &p->ring_in}) {
    while (!r->live.empty()) {
      Region& f = r->live.front();
      if (!f.recorded || p->event_query(f.freed) != hipSuccess) break;
      put_event(p, f.freed);
      r->live.pop_front();
    }
  }
  p->alloc.reap(p->pack_done_seq, p->scat_done_seq);
}

Op* find_op(std::deque<OpRef>& dq, uint64_t seq) {
  if (dq.empty() || seq < dq.front()->seq) return nullptr;
  size_t i = (size_t)(seq - dq.front()->seq);
  return i < dq.size() ? dq[i].get() : nullptr;
}

// Host wait for one op (lock held by caller; short waits only on rare paths).
int32_t host_wait_op(kv_pool* p, const OpRef& op_ref) {
  const OpRef op = op_ref;  // the caller's reference may point into the request table
  if (!op || op->all_done || p->plan) return KV_OK;
  int32_t rc = wait_issued(p, op);  // drops the lock while a held-back swap-out is handed over
  if (rc) return rc;
  if (op->done) HIP_TRY(hipEventSynchronize(op->done));
  reap(p);
  return KV_OK;
}

// ---------------------------------------------------------------- engine
// base + off; a plan-only pool has no memory behind its bases (null stays null)
static inline char* at(char* base, int64_t off) { return base ? base + off : nullptr; }

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

// One pack launch over m blocks and the planes [p0, p0 + np) (np = 0: all planes); staging
// holds [m][np][C].
// op (may be null) and op_bytes: the swap this launch belongs to and the bytes it moves in all.
// The pack launches of a swap of defer_min_bytes or more carry begin and end events of their own
// also when nobody reads them.  Measured on config 3 (a swap-out and a swap-in per step beside
// GEMMs), pools without KV_FLAG_PROFILE: with plain launches 90.8 GB/s, median 38.4 / p99 65 ms when
// the step's swap-in is issued first, but 79.3 GB/s and 44.5 / 97.8 ms when the swap-out is, and in a
// plain loop of one swap-in and one swap-out at a time the two directions took turns on the link
// (56.6 GB/s in all, until a hipStreamSynchronize of the pool's streams).  With the events on the
// launches 91.9 GB/s and 37 / 69 ms in either order, and 95.6 GB/s in the plain loop.  Events around
// the copies instead change nothing.  A launch that has events gets a completion signal of its own,
// which is presumably what the copy that follows it then waits for; what the runtime does without
// one is not visible from here.  Small swaps keep the plain launch: the events cost a swap-out on its
// own 17-20 us and a swap-in 8 us, and pay for a pair issued together from about 8 MiB each.
int32_t launch_pack(kv_pool* p, bool scatter, char* staging, const Move* mv, int64_t m,
                    int32_t p0 = 0, int32_t np = 0, Op* op = nullptr, int64_t op_bytes = 0) {
  hipStream_t s = scatter ? p->s_scat : p->s_pack;
  (scatter ? p->st.scatter_launches : p->st.gather_launches)++;
  if (p->plan) return KV_OK;
  if (np == 0) np = p->P;
  KvPackArgs a;
  a.pool = p->gpu + (int64_t)p0 * p->N * p->C;
  a.staging = staging;
  a.plane_stride = p->N * p->C;
  a.C = (uint32_t)p->C;
  a.P = (uint32_t)np;
  a.m = (uint32_t)m;
  a.tiles_per_chunk = a.n_tiles = a.xcd_blocks = 0;
  for (int64_t i = 0; i < m; ++i) a.table[i] = mv[i].phys;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (p->profile) {
    int32_t rc = get_timing_event(p, &e0);
    if (rc) return rc;
    rc = get_timing_event(p, &e1);
    if (rc) return rc;
    p->prof.push_back({scatter ? 1 : 0, m * np * p->C, e0, e1});
  } else if (op && p->launch_events && op_bytes >= p->defer_min) {
    int32_t rc = get_timing_event(p, &e0);
    if (rc) return rc;
    op->timed.push_back(e0);
    rc = get_timing_event(p, &e1);
    if (rc) return rc;
    op->timed.push_back(e1);
  }
  HIP_TRY(kv_launch_pack(scatter, a, p->unroll, p->variant, p->grid, s, e0, e1));
  return KV_OK;
}

// Copies of one ring slot.  A maximal run of moves whose host records are adjacent is one
// contiguous copy; consecutive runs of EQUAL length whose host positions are a constant
// positive stride apart (an arithmetic progression of records; order_for_strided_copies
// arranges move lists that way) go out as the rows of ONE 2-D copy: the copy engines take
// about 9 us per copy whatever its shape, so scattered block records (a delta swap-out's
// dirty blocks, Section 3.3) cost a third of the dispatches.  Measured on MI355X, 2 MiB
// records far apart on the host: 45.5 GB/s one by one, 50.6 / 52.5 / 53.6 / 55.2 GB/s as
// 2-D copies of 2 / 3 / 4 / 8 rows, for pitches up to 1 GiB; the same 13 us per copy for rows
// of 32 KiB, 4 MiB, 12.5 MiB and 16 MiB.  Rows wider than 16 MiB (not measured, and efficient
// on their own) always travel as plain copies.  Every copy is cut at copy_chunk bytes.

void plan_copies(const Move* mv, int64_t m, int64_t R, int64_t copy_chunk, bool strided, std::vector<CopyDesc>* out) {
  auto run_end = [&](int64_t i) {  // last move of the maximal run of adjacent records that starts at i
    int64_t j = i;
    while (j + 1 < m && mv[j + 1].host_off == mv[j].host_off + R) ++j;
    return j;
  };
  int64_t i = 0;
  while (i < m) {
    const int64_t j = run_end(i);
    const int64_t len = j - i + 1, width = len * R;
    // further rows: runs of the same length, a constant stride apart
    int64_t rows = 1, pitch = 0;
    if (strided && width < copy_chunk && width <= KV_MAX_STRIDED_WIDTH) {
      int64_t nx = j + 1;
      while (nx < m && (rows + 1) * width <= copy_chunk) {
        if (run_end(nx) - nx + 1 != len) break;
        const int64_t d = mv[nx].host_off - mv[nx - len].host_off;
        if (rows == 1) {
          if (d < width || d > KV_MAX_COPY_PITCH) break;
          pitch = d;
        } else if (d != pitch) {
          break;
        }
        ++rows;
        nx += len;
      }
    }
    if (rows > 1) {
      out->push_back({mv[i].host_off, i * R, width, rows, pitch});
      i += rows * len;
      continue;
    }
    for (int64_t o = 0; o < width; o += copy_chunk)
      out->push_back({mv[i].host_off + o, i * R + o, std::min(copy_chunk, width - o), 1, 0});
    i = j + 1;
  }
}

// One copy of a plan, on stream s.
static int32_t issue_one(kv_pool* p, bool to_host, char* slot, const CopyDesc& c, hipStream_t s) {
  char* h = p->host + c.host_off;
  char* d = slot + c.slot_off;
  if (c.rows > 1) {
    if (to_host)
      HIP_TRY(hipMemcpy2DAsync(h, (size_t)c.pitch, d, (size_t)c.width, (size_t)c.width, (size_t)c.rows,
                               hipMemcpyDeviceToHost, s));
    else
      HIP_TRY(hipMemcpy2DAsync(d, (size_t)c.width, h, (size_t)c.pitch, (size_t)c.width, (size_t)c.rows,
                               hipMemcpyHostToDevice, s));
  } else if (to_host) {
    HIP_TRY(hipMemcpyAsync(h, d, (size_t)c.width, hipMemcpyDeviceToHost, s));
  } else {
    HIP_TRY(hipMemcpyAsync(d, h, (size_t)c.width, hipMemcpyHostToDevice, s));
  }
  return KV_OK;
}

// KV_FLAG_SECOND_LANE: the scattered records of a held-back swap-out as plain copies, every other one
// on `lane2`, the host-to-device stream, whose copy engine has nothing to do while no swap-in is in
// flight.  A copy engine spends about 9 us between two copies; two engines spend them in turn.
// Measured (2 MiB records, a fifth of a 400-block image dirty): 45.6 GB/s as plain copies on one
// stream, 50.8 as 2-D copies on one stream (the default), 52-53 this way.  2-D copies themselves do
// not run side by side on two streams (45.5 GB/s on one or on two), and a second stream of the same
// direction shares the first one's engine, so it has to be this stream and plain copies.
// What makes the second stream use another engine is the runtime's to decide; what was seen is that a
// stream with nothing outstanding takes an engine that is free at that moment and then stays on it.
// So the second lane is synchronised first (its earlier copies are long done) and gets its first
// copy only when the own lane's first copy has finished and its second one is running.  Without
// that the second lane ended up on the own lane's engine in whole processes (46 GB/s).
// The own stream is made to wait for the second lane's last copy, so what is recorded on it
// afterwards covers both; the events used go to *aux.  Called by the copy thread only: the copies
// depend on nothing that still runs, and the caller has seen that no swap-in is in flight.
static int32_t issue_two_lanes(kv_pool* p, char* slot, const std::vector<CopyDesc>& plan, hipStream_t lane2,
                               std::vector<hipEvent_t>* aux) {
  int32_t rc;
  hipEvent_t first_done, hop;
  if ((rc = get_event(p, &first_done))) return rc;
  aux->push_back(first_done);
  if ((rc = get_event(p, &hop))) return rc;
  aux->push_back(hop);
  const hipStream_t own = p->s_d2h;
  if ((rc = issue_one(p, true, slot, plan[0], own))) return rc;
  HIP_TRY(hipEventRecord(first_done, own));
  if ((rc = issue_one(p, true, slot, plan[2], own))) return rc;
  HIP_TRY(hipStreamSynchronize(lane2));
  HIP_TRY(hipEventSynchronize(first_done));
  for (size_t k = 1; k < plan.size(); ++k) {
    if (k == 2) continue;
    if ((rc = issue_one(p, true, slot, plan[k], (k & 1) ? lane2 : own))) return rc;
  }
  HIP_TRY(hipEventRecord(hop, lane2));
  HIP_TRY(hipStreamWaitEvent(own, hop, 0));
  p->st.d2h_copies += (int64_t)plan.size();
  p->st.second_lane_copies += (int64_t)plan.size() / 2;
  return KV_OK;
}

int32_t issue_copies(kv_pool* p, bool to_host, char* slot, const Move* mv, int64_t m, hipStream_t lane2 = nullptr,
                     std::vector<hipEvent_t>* aux = nullptr) {
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
  std::vector<CopyDesc> plan;
  if (lane2 && to_host && !p->plan && m * p->R <= KV_SECOND_LANE_MAX_PIECE_BYTES) {
    // worth two lanes: several plain copies of a few MiB each (the sizes measured)
    plan_copies(mv, m, p->R, p->copy_chunk, false, &plan);
    const int64_t n = (int64_t)plan.size();
    if (n >= KV_SECOND_LANE_MIN_COPIES && m * p->R >= n * KV_SECOND_LANE_MIN_AVG_BYTES &&
        m * p->R <= n * KV_SECOND_LANE_MAX_AVG_BYTES) {
      int32_t rc = issue_two_lanes(p, slot, plan, lane2, aux);
      if (rc) return rc;
      if (e1) HIP_TRY(hipEventRecord(e1, s));
      return KV_OK;
    }
    plan.clear();
  }
  plan_copies(mv, m, p->R, p->copy_chunk, p->strided_copies, &plan);
  for (const CopyDesc& c : plan) {
    (to_host ? p->st.d2h_copies : p->st.h2d_copies)++;
    if (c.rows > 1) p->st.strided_copies++;
    if (p->plan) continue;
    int32_t rc = issue_one(p, to_host, slot, c, s);
    if (rc) return rc;
  }
  if (e1) HIP_TRY(hipEventRecord(e1, s));
  return KV_OK;
}

// Records `ev` so that it fires when the work enqueued so far on `from` is done, but ON stream
// `on`: completion events of one direction are all recorded on one stream (packed: s_pack,
// swap-out done: s_d2h, swap-in done: s_scat), whatever stream a path did its work on, so they
// fire in issue order and waiting for the newest op of a set covers the older ones.
int32_t record_via(kv_pool* p, hipEvent_t ev, hipStream_t from, hipStream_t on, const OpRef& op) {
  if (p->plan || !ev) return KV_OK;
  if (from != on) {
    int32_t rc;
    hipEvent_t hop;
    if ((rc = get_event(p, &hop))) return rc;
    op->aux.push_back(hop);
    HIP_TRY(hipEventRecord(hop, from));
    HIP_TRY(hipStreamWaitEvent(on, hop, 0));
  }
  HIP_TRY(hipEventRecord(ev, on));
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
// An event another stream has just been told to wait for is not recycled at once: it goes to
// the claiming op's list (`retired`) and back to the pool when that op is done, so nothing can
// record it again while the wait is still queued.
template <class Flush>
int32_t ring_claim(kv_pool* p, ByteRing* r, int64_t len, uint64_t op_seq, hipStream_t producer,
                   Flush&& flush, std::vector<hipEvent_t>* retired, Region** out) {
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
      if (f.freed) retired->push_back(f.freed);
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

// Copies of one gathered piece (moves [first, first + count) at ring offset off) to the host, and
// the event that gives its ring region back.
static int32_t drain_piece(kv_pool* p, ByteRing& r, uint64_t op_seq, const Move* mv, int64_t first,
                           int64_t count, int64_t off, hipStream_t lane2 = nullptr,
                           std::vector<hipEvent_t>* aux = nullptr) {
  int32_t rc;
  if ((rc = issue_copies(p, true, at(r.base, off), mv + first, count, lane2, aux))) return rc;
  for (Region& g : r.live)
    if (g.off == off && g.op_seq == op_seq && !g.recorded) {
      if ((rc = record(p, g.freed, p->s_d2h))) return rc;
      g.recorded = true;
    }
  return KV_OK;
}

// The copy thread of a pool (none with KV_FLAG_NO_DEFER_COPIES).  A device-to-host copy that is handed to
// the runtime while the gather it follows has not finished waits for it inside a copy engine's
// queue, and a host-to-device copy of another request that the runtime puts on the same engine
// afterwards waits behind it (seen in a serving loop beside GEMMs: a swap-in issued right after a
// swap-out finished only when two queued swap-outs had drained).  Here a swap-out's copies reach
// the runtime only when nothing holds them back any more: this thread waits on the host for
// each piece's gathers, then enqueues the piece's copies, and after the last piece the op's
// completion event.  Until then the op counts as not issued: nothing polls or waits for its
// completion event (wait_issued), and the next swap-out waits for this one's hand-over.
static void copy_thread_main(kv_pool* p) {
  (void)hipSetDevice(p->device);
  std::unique_lock<std::mutex> lk(p->mu);
  for (;;) {
    p->cv_job.wait(lk, [&] { return p->copy_thread_stop || !p->jobs.empty(); });
    if (p->jobs.empty()) return;
    DeferredOut job = std::move(p->jobs.front());
    p->jobs.pop_front();
    int32_t rc = KV_OK;
    auto note = [&](int32_t r2) {
      if (r2 && !rc) rc = r2;
    };
    for (const DeferredPiece& q : job.pieces) {
      lk.unlock();
      const hipError_t e = hipEventSynchronize(q.ready);
      lk.lock();
      if (e != hipSuccess) note(fail(KV_EHIP, "copy thread: hipEventSynchronize: %s", hipGetErrorString(e)));
      note(stream_wait(p, p->s_d2h, q.ready));  // already complete: costs nothing, and keeps the order on the device explicit
      // KV_FLAG_SECOND_LANE: while no swap-in is in flight the host-to-device stream may carry every
      // other copy of a piece of scattered records (issue_two_lanes)
      hipStream_t lane2 = nullptr;
      if (p->second_lane) {
        reap(p);
        if (p->ops_in.empty()) lane2 = p->s_h2d;
      }
      note(drain_piece(p, p->ring_out, job.op->seq, job.mv.data(), q.first, q.count, q.off, lane2, &job.op->aux));
    }
    note(record(p, job.op->done, p->s_d2h));
    job.op->issued = true;
    if (rc && !p->copy_thread_rc) {
      p->copy_thread_rc = rc;
      p->copy_thread_err = g_err;
    }
    --p->deferred_pending;
    p->cv_issued.notify_all();
  }
}

int32_t wait_issued(kv_pool* p, const OpRef& op) {
  if (op && !op->issued) p->cv_issued.wait(p->mu, [&] { return op->issued; });
  if (p->copy_thread_rc) {
    g_err = p->copy_thread_err;
    return p->copy_thread_rc;
  }
  return KV_OK;
}

int32_t wait_all_issued(kv_pool* p) {
  if (p->deferred_pending > 0) p->cv_issued.wait(p->mu, [&] { return p->deferred_pending == 0; });
  if (p->copy_thread_rc) {
    g_err = p->copy_thread_err;
    return p->copy_thread_rc;
  }
  return KV_OK;
}

// Bytes of the out ring that a new swap-out can claim before its claims would have to evict a
// region whose copies have not been enqueued yet (regions are claimed and retired in ring
// order, so those are the newest ones).  A piece that does not fit before the end of the ring
// skips the tail: one piece is held in reserve for that.
int64_t out_ring_room(kv_pool* p) {
  const ByteRing& r = p->ring_out;
  const int64_t piece = r.piece_blocks * p->R;
  for (const Region& g : r.live) {
    if (g.recorded) continue;
    const int64_t ahead = g.off >= r.head ? g.off - r.head : r.cap - r.head + g.off;
    return std::max<int64_t>(0, ahead - piece);
  }
  return r.cap - piece;
}

void stop_copy_thread(kv_pool* p, std::unique_lock<std::mutex>& lk) {
  (void)wait_all_issued(p);
  if (!p->copy_thread.joinable()) return;
  p->copy_thread_stop = true;
  p->cv_job.notify_all();
  lk.unlock();
  p->copy_thread.join();
  lk.lock();
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
    hipEvent_t ready;  // held-back copies only: recorded behind this piece's gathers
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
    for (const Pending& q : pending)
      if ((rc2 = drain_piece(p, r, op->seq, mv.data(), q.first, q.count, q.off))) return rc2;
    pending.clear();
    return KV_OK;
  };
  const bool defer = p->defer_copies && !p->plan && m * p->R >= p->defer_min;
  for (int64_t i = 0; i < m; i += r.piece_blocks) {
    const int64_t mp = std::min(r.piece_blocks, m - i);
    Region* g;
    if ((rc = ring_claim(p, &r, mp * p->R, op->seq, p->s_pack, flush, &op->aux, &g))) return rc;
    const int64_t off = g->off;
    for (int64_t k = 0; k < mp; k += p->launch_blocks) {
      int64_t ml = std::min<int64_t>(p->launch_blocks, mp - k);
      if ((rc = launch_pack(p, false, at(r.base, off + k * p->R), &mv[(size_t)(i + k)], ml, 0, 0, op.get(), m * p->R)))
        return rc;
    }
    hipEvent_t piece_ready = nullptr;
    if (defer) {
      if ((rc = get_event(p, &piece_ready))) return rc;
      op->aux.push_back(piece_ready);
      if ((rc = record(p, piece_ready, p->s_pack))) return rc;
    }
    pending.push_back({i, mp, off, piece_ready});
    // gathers and copies on streams of their own: a piece's copies start as soon as its gather is
    // done, and the following gathers run under them (held-back copies: the copy thread does that)
    if (!defer && p->s_pack != p->s_d2h && (rc = flush())) return rc;
  }
  if ((rc = record(p, op->packed, p->s_pack))) return rc;
  p->st.bytes_out += m * p->R;
  p->st.blocks_out += m;
  if (defer && !pending.empty()) {
    // the copies, the regions' release and the completion event are the copy thread's to enqueue,
    // piece by piece, once the host has seen each piece's gathers finish
    DeferredOut job;
    job.op = op;
    job.mv = mv;
    for (const Pending& q : pending) job.pieces.push_back({q.first, q.count, q.off, q.ready});
    op->deferred = true;
    p->jobs.push_back(std::move(job));
    ++p->deferred_pending;
    if (!p->copy_thread.joinable()) p->copy_thread = std::thread(copy_thread_main, p);
    p->cv_job.notify_one();
    return KV_OK;
  }
  if ((rc = flush())) return rc;
  if (m == 0 && (rc = stream_wait(p, p->s_d2h, op->packed))) return rc;
  if ((rc = record(p, op->done, p->s_d2h))) return rc;
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
  // What the scatters have to wait for (the caller's compute, gathers that still read the target
  // blocks) is put in front of the first scatter, not in front of the copies: with one stream per
  // direction the first piece's copy into staging then runs while that work finishes.
  bool scatter_ordered = false;
  auto order_scatters = [&]() -> int32_t {
    if (scatter_ordered) return KV_OK;
    scatter_ordered = true;
    int32_t rc2;
    if ((rc2 = order_after_compute(p, p->s_scat))) return rc2;
    for (hipEvent_t e : pre_scat)
      if ((rc2 = stream_wait(p, p->s_scat, e))) return rc2;
    return KV_OK;
  };
  ByteRing& r = p->ring_in;
  const int64_t m = (int64_t)mv.size();
  auto no_flush = []() -> int32_t { return KV_OK; };  // every region is closed before the next claim
  for (int64_t i = 0; i < m; i += r.piece_blocks) {
    const int64_t mp = std::min(r.piece_blocks, m - i);
    Region* g;
    if ((rc = ring_claim(p, &r, mp * p->R, op->seq, p->s_h2d, no_flush, &op->aux, &g))) return rc;
    char* sb = at(r.base, g->off);
    if ((rc = issue_copies(p, false, sb, &mv[(size_t)i], mp))) return rc;
    hipEvent_t ready;
    if ((rc = get_event(p, &ready))) return rc;
    if (ready) op->aux.push_back(ready);
    if ((rc = record(p, ready, p->s_h2d))) return rc;
    if ((rc = stream_wait(p, p->s_scat, ready))) return rc;
    if ((rc = order_scatters())) return rc;
    for (int64_t k = 0; k < mp; k += p->launch_blocks) {
      int64_t ml = std::min<int64_t>(p->launch_blocks, mp - k);
      if ((rc = launch_pack(p, true, at(sb, k * p->R), &mv[(size_t)(i + k)], ml, 0, 0, op.get(), m * p->R))) return rc;
    }
    if ((rc = record(p, g->freed, p->s_scat))) return rc;
    g->recorded = true;
  }
  if ((rc = order_scatters())) return rc;  // an empty move list still completes in order
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

// Layer-wise swap-in (the layer-wise asynchronous swapping of earlier systems that Section
// 2.2, Challenge #2, discusses): the request's KV arrives in steps of `step` layers, lowest
// layers first, and an event per step lets the consumer start on layer l while the layers
// above it are still on the link.  In the block-major host image the K and V planes of
// `step` consecutive layers are one contiguous slice of 2*step*C bytes in every record, so a
// step is one 2-D copy per run of adjacent records (rows = blocks, R bytes apart on the
// host, packed in staging) followed by a scatter over that plane range.
int32_t enqueue_in_layers(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre_copy,
                          const std::vector<hipEvent_t>& pre_scat, const OpRef& op, int32_t step) {
  int32_t rc;
  for (hipEvent_t e : pre_copy)
    if ((rc = stream_wait(p, p->s_h2d, e))) return rc;
  if ((rc = order_after_compute(p, p->s_scat))) return rc;
  for (hipEvent_t e : pre_scat)
    if ((rc = stream_wait(p, p->s_scat, e))) return rc;
  if (mv.empty())
    for (hipEvent_t e : pre_copy)
      if ((rc = stream_wait(p, p->s_scat, e))) return rc;
  ByteRing& r = p->ring_in;
  const int64_t m = (int64_t)mv.size();
  const int32_t L = p->P / 2;
  auto no_flush = []() -> int32_t { return KV_OK; };
  op->layer_step = step;
  for (int32_t l0 = 0; l0 < L; l0 += step) {
    const int32_t np = 2 * std::min(step, L - l0), p0 = 2 * l0;
    const int64_t slice = (int64_t)np * p->C;
    const int64_t piece_blocks = std::max<int64_t>(1, r.piece_blocks * p->R / slice);
    const int64_t rows_per_copy = std::max<int64_t>(1, p->copy_chunk / slice);
    for (int64_t i = 0; i < m; i += piece_blocks) {
      const int64_t mp = std::min(piece_blocks, m - i);
      Region* g;
      if ((rc = ring_claim(p, &r, mp * slice, op->seq, p->s_h2d, no_flush, &op->aux, &g))) return rc;
      char* sb = at(r.base, g->off);
      hipEvent_t e0 = nullptr, e1 = nullptr;
      if (p->profile && !p->plan) {
        if ((rc = get_timing_event(p, &e0))) return rc;
        if ((rc = get_timing_event(p, &e1))) return rc;
        p->prof.push_back({3, mp * slice, e0, e1});
        HIP_TRY(hipEventRecord(e0, p->s_h2d));
      }
      int64_t a = 0;
      while (a < mp) {
        int64_t b = a;
        while (b + 1 < mp && b + 1 - a < rows_per_copy &&
               mv[(size_t)(i + b + 1)].host_off == mv[(size_t)(i + b)].host_off + p->R)
          ++b;
        p->st.h2d_copies++;
        if (!p->plan)
          HIP_TRY(hipMemcpy2DAsync(sb + a * slice, (size_t)slice,
                                   p->host + mv[(size_t)(i + a)].host_off + (int64_t)p0 * p->C, (size_t)p->R,
                                   (size_t)slice, (size_t)(b - a + 1), hipMemcpyHostToDevice, p->s_h2d));
        a = b + 1;
      }
      if (e1) HIP_TRY(hipEventRecord(e1, p->s_h2d));
      hipEvent_t ready;
      if ((rc = get_event(p, &ready))) return rc;
      if (ready) op->aux.push_back(ready);
      if ((rc = record(p, ready, p->s_h2d))) return rc;
      if ((rc = stream_wait(p, p->s_scat, ready))) return rc;
      for (int64_t k = 0; k < mp; k += p->launch_blocks) {
        int64_t ml = std::min<int64_t>(p->launch_blocks, mp - k);
        if ((rc = launch_pack(p, true, at(sb, k * slice), &mv[(size_t)(i + k)], ml, p0, np))) return rc;
      }
      if ((rc = record(p, g->freed, p->s_scat))) return rc;
      g->recorded = true;
    }
    hipEvent_t landed;
    if ((rc = get_event(p, &landed))) return rc;
    op->layer_ev.push_back(landed);
    if ((rc = record(p, landed, p->s_scat))) return rc;
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
      char* h = at(p->host, mv[(size_t)i].host_off + (int64_t)pl * p->C);
      char* d = at(p->gpu, ((int64_t)pl * p->N + mv[(size_t)i].phys) * p->C);
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
  if (to_host) {
    if ((rc = record_via(p, op->packed, s, p->s_pack, op))) return rc;
    if ((rc = record(p, op->done, s))) return rc;
  } else {
    if ((rc = record_via(p, op->done, s, p->s_scat, op))) return rc;
  }
  (to_host ? p->st.bytes_out : p->st.bytes_in) += m * p->R;
  (to_host ? p->st.blocks_out : p->st.blocks_in) += m;
  return KV_OK;
}

// Swap-in straight from the pinned image (KV_FLAG_MAPPED_SWAP_IN): one persistent kernel per
// 440 blocks reads the host records over the link and writes the pool; no staging, no copy
// engine, no per-run copies - fragmented images and partial swap-ins cost the same as
// contiguous ones.
int32_t enqueue_in_mapped(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                          const OpRef& op, int32_t layer_step) {
  int32_t rc;
  hipStream_t s = p->s_scat;
  if ((rc = order_after_compute(p, s))) return rc;
  for (hipEvent_t e : pre)
    if ((rc = stream_wait(p, s, e))) return rc;
  const int64_t m = (int64_t)mv.size();
  const int32_t L = p->P / 2;
  // layer-wise: one launch per step of layers over that slice of every record, and an event
  // behind it; otherwise a single step over all planes
  const int32_t step = layer_step > 0 ? layer_step : L;
  op->layer_step = layer_step;
  for (int32_t l0 = 0; l0 < L; l0 += step) {
    const int32_t np = 2 * std::min(step, L - l0), p0 = 2 * l0;
    for (int64_t i = 0; i < m; i += KV_MAX_MAPPED_BLOCKS) {
      const int64_t ml = std::min<int64_t>(KV_MAX_MAPPED_BLOCKS, m - i);
      p->st.scatter_launches++;
      if (p->plan) continue;
      KvMappedArgs a;
      a.pool = p->gpu + (int64_t)p0 * p->N * p->C;
      a.host = p->host_dev + (int64_t)p0 * p->C;
      a.plane_stride = p->N * p->C;
      a.R = p->R;
      a.C = (uint32_t)p->C;
      a.P = (uint32_t)np;
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
        p->prof.push_back({4, ml * np * p->C, e0, e1});
      }
      HIP_TRY(kv_launch_mapped(false, a, p->mapped_grid, s, e0, e1));
    }
    if (layer_step > 0) {
      hipEvent_t landed;
      if ((rc = get_event(p, &landed))) return rc;
      op->layer_ev.push_back(landed);
      if ((rc = record(p, landed, s))) return rc;
    }
  }
  if ((rc = record(p, op->done, s))) return rc;
  p->st.bytes_in += m * p->R;
  p->st.blocks_in += m;
  return KV_OK;
}

// Swap-out straight into the pinned image (KV_FLAG_MAPPED_SWAP_OUT, small requests): one
// launch per 440 blocks reads the pool and stores the records to host memory.  The gather is
// the transfer, so the request's GPU blocks are reusable exactly when the swap-out is done.
int32_t enqueue_out_mapped(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                           const OpRef& op) {
  int32_t rc;
  hipStream_t s = p->s_pack;
  if ((rc = order_after_compute(p, s))) return rc;
  for (hipEvent_t e : pre)
    if ((rc = stream_wait(p, s, e))) return rc;
  const int64_t m = (int64_t)mv.size();
  for (int64_t i = 0; i < m; i += KV_MAX_MAPPED_BLOCKS) {
    const int64_t ml = std::min<int64_t>(KV_MAX_MAPPED_BLOCKS, m - i);
    p->st.gather_launches++;
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
      p->prof.push_back({5, ml * p->R, e0, e1});
    }
    HIP_TRY(kv_launch_mapped(true, a, p->mapped_grid, s, e0, e1));
  }
  if ((rc = record(p, op->packed, s))) return rc;
  if ((rc = record_via(p, op->done, s, p->s_d2h, op))) return rc;
  p->st.bytes_out += m * p->R;
  p->st.blocks_out += m;
  return KV_OK;
}

// Arranges a move list for issue_copies: runs of adjacent host records of equal length whose
// positions form an arithmetic progression are placed next to each other, so that each
// progression becomes one 2-D copy.  The order of a move list is free (it fixes the order of
// the records in staging, nothing else).  Greedy: runs are grouped by length; inside a group,
// sorted by position, the first remaining run starts a progression whose stride is the one,
// among the distances to the next few runs, that yields the longest chain.  O(n log n) for n
// runs; lists with fewer than three runs are left alone.
void order_for_strided_copies(kv_pool* p, std::vector<Move>& mv) {
  if (!p->strided_copies || mv.size() < 3) return;
  struct Run {
    int64_t first, len, rec;  // index in mv, blocks, host record of the first block
  };
  std::vector<Run> runs;
  const int64_t m = (int64_t)mv.size();
  for (int64_t i = 0; i < m;) {
    int64_t j = i;
    while (j + 1 < m && mv[(size_t)j + 1].host_off == mv[(size_t)j].host_off + p->R) ++j;
    runs.push_back({i, j - i + 1, mv[(size_t)i].host_off / p->R});
    i = j + 1;
  }
  if (runs.size() < 3) return;
  // groups of equal length, longest runs first; positions ascending inside a group
  std::vector<size_t> order(runs.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = i;
  std::sort(order.begin(), order.end(), [&](size_t a, size_t b) {
    return runs[a].len != runs[b].len ? runs[a].len > runs[b].len : runs[a].rec < runs[b].rec;
  });
  std::vector<Move> out;
  out.reserve(mv.size());
  auto emit = [&](const Run& r) {
    for (int64_t k = 0; k < r.len; ++k) out.push_back(mv[(size_t)(r.first + k)]);
  };
  constexpr int CANDIDATES = 8;
  for (size_t g0 = 0; g0 < order.size();) {
    size_t g1 = g0;
    while (g1 < order.size() && runs[order[g1]].len == runs[order[g0]].len) ++g1;
    const size_t n = g1 - g0;
    const int64_t len = runs[order[g0]].len;
    const int64_t max_rows = std::max<int64_t>(1, p->copy_chunk / (len * p->R));
    const int64_t max_stride = KV_MAX_COPY_PITCH / p->R;
    if (n < 3 || max_rows < 2 || len * p->R > KV_MAX_STRIDED_WIDTH) {
      for (size_t a = g0; a < g1; ++a) emit(runs[order[a]]);
      g0 = g1;
      continue;
    }
    std::vector<int64_t> pos(n);
    std::vector<uint8_t> taken(n, 0);
    for (size_t a = 0; a < n; ++a) pos[a] = runs[order[g0 + a]].rec;
    auto find = [&](int64_t x) -> int64_t {  // index of the untaken run at position x, or -1
      auto it = std::lower_bound(pos.begin(), pos.end(), x);
      if (it == pos.end() || *it != x) return -1;
      const size_t k = (size_t)(it - pos.begin());
      return taken[k] ? -1 : (int64_t)k;
    };
    std::vector<int64_t> chain, best;
    for (size_t a = 0; a < n; ++a) {
      if (taken[a]) continue;
      best.assign(1, (int64_t)a);
      int tried = 0;
      for (size_t b = a + 1; b < n && tried < CANDIDATES; ++b) {
        if (taken[b]) continue;
        const int64_t d = pos[b] - pos[a];
        if (d > max_stride) break;
        if (d < len) continue;  // rows may not overlap
        ++tried;
        chain.assign(1, (int64_t)a);
        int64_t k = (int64_t)b;
        while (k >= 0 && (int64_t)chain.size() < max_rows) {
          chain.push_back(k);
          k = find(pos[(size_t)k] + d);
        }
        if (chain.size() > best.size()) best = chain;
      }
      for (int64_t k : best) {
        taken[(size_t)k] = 1;
        emit(runs[order[g0 + (size_t)k]]);
      }
    }
    g0 = g1;
  }
  mv.swap(out);
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

}  // namespace kvi
