// Reuse map of the KV-swap library: table validation, the pinned host arena and the host
// images that live in it, eviction, and the selection of the blocks a swap moves (FastSwitch,
// arXiv 2411.18424, Section 3.3: keep the CPU copy, send only what it lacks, track which
// parts were contaminated, reserve room next to the copy for the next turn).

#include "kv_pool.hpp"

namespace kvi {

namespace {

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

}  // namespace

void arena_give(kv_pool* p, const std::vector<Extent>& ext) {
  for (const Extent& e : ext)
    if (e.cap > 0) p->arena.insert(e.off, e.cap);
}

namespace {

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

}  // namespace


int32_t do_swap_out(kv_pool* p, std::vector<OutItem>& items, int32_t* out_n_moved, int direct) {
  int32_t rc;
  // Swap-outs whose copies are still held back keep their regions of the out ring open, and their
  // completion events do not exist on the device yet.  This call may be enqueued behind them if
  // it follows none of them on its own requests and fits the ring without reaching their regions;
  // otherwise it waits, on the host, for their hand-over.
  if (p->deferred_pending > 0) {
    int64_t need = 0;
    bool own = false;
    for (const OutItem& it : items) {
      need += std::max<int64_t>(it.n, 0) * p->R;
      auto f = p->reqs.find(it.req);
      own |= f != p->reqs.end() && f->second.last && !f->second.last->issued;
    }
    if (own || need > out_ring_room(p)) {
      if ((rc = wait_all_issued(p))) return rc;
    } else if (p->copy_thread_rc) {
      return wait_all_issued(p);  // reports the copy thread's error
    }
  }
  reap(p);
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
  // 3. an image that is rebuilt gives its old extents back to the arena; an unfinished op of
  //    the request may still read or write them.  Wait for it now, before this call's op
  //    exists: completion polling must never meet an op whose events are not recorded yet.
  for (OutItem& it : items) {
    if (!it.fresh) continue;
    auto f = p->reqs.find(it.req);
    if (f == p->reqs.end() || !f->second.has_image) continue;
    if ((rc = host_wait_op(p, f->second.last))) {
      undo(items.size());
      return rc;
    }
  }
  // 4. commit: images, reuse map, move list
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
      if (q.has_image) arena_give(p, im.ext);  // its last op has finished (step 3)
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
  if (direct)
    rc = enqueue_direct(p, true, mv, pre, op, direct == 2);
  else if (p->mapped_out && (p->mapped_out_max == 0 || (int64_t)mv.size() <= p->mapped_out_max))
    rc = enqueue_out_mapped(p, mv, pre, op);
  else {
    order_for_strided_copies(p, mv);
    rc = enqueue_out(p, mv, pre, op);
  }
  op->packed_recorded = true;
  if (!op->deferred) op->issued = true;  // also after a failed enqueue, so that polling does not stop here for ever
  return rc;
}


int32_t do_swap_in(kv_pool* p, std::vector<InItem>& items, int32_t* out_n_moved, int direct,
                   int32_t layer_step) {
  int32_t rc;
  // a swap-in follows its request's last op through that op's completion event: if the op is a
  // swap-out whose copies are still held back, the event does not exist on the device yet.
  // Swap-ins of other requests go ahead - that is what holding the copies back is for.
  for (const InItem& it : items) {
    auto f = p->reqs.find(it.req);
    if (f == p->reqs.end() || !f->second.last) continue;
    const OpRef last = f->second.last;  // the lock is dropped during the wait
    if ((rc = wait_issued(p, last))) return rc;
  }
  reap(p);
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
  uint64_t max_reader = 0, max_writer = 0;
  for (InItem& it : items) {
    Req& q = p->reqs[it.req];
    for (int32_t j = 0; j < it.n; ++j) {
      if (it.resident && it.resident[j]) continue;
      int32_t b = it.table[j];
      mv.push_back({q.img.rec[(size_t)j] * p->R, b});
      max_writer = std::max(max_writer, p->writer_seq[(size_t)b]);
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
  if (max_writer > p->scat_done_seq) {
    // an earlier swap-in into these blocks is still in flight: write after it, whatever
    // stream it runs on (the paths of this library use more than one)
    if (Op* w = find_op(p->ops_in, max_writer))
      if (w->done) pre_scat.push_back(w->done);
  }
  if (out_n_moved) *out_n_moved = (int32_t)mv.size();
  if (direct) {
    pre_copy.insert(pre_copy.end(), pre_scat.begin(), pre_scat.end());
    rc = enqueue_direct(p, false, mv, pre_copy, op, direct == 2);
  } else if (p->mapped_in) {
    pre_copy.insert(pre_copy.end(), pre_scat.begin(), pre_scat.end());
    rc = enqueue_in_mapped(p, mv, pre_copy, op, layer_step);
  } else if (layer_step > 0) {
    rc = enqueue_in_layers(p, mv, pre_copy, pre_scat, op, layer_step);
  } else {
    order_for_strided_copies(p, mv);
    rc = enqueue_in(p, mv, pre_copy, pre_scat, op);
  }
  op->issued = true;
  return rc;
}

}  // namespace kvi
