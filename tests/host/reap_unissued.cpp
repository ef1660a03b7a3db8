// Host-only unit test of the completion polling (kvi::reap) of the KV-swap library's engine.
//
// The HIP runtime reports an event that was never recorded - or that was recycled from an
// earlier, finished op - as complete.  An op that exists but whose events have not been
// recorded yet (it is still being enqueued) must therefore never be looked at by the
// polling, or it would be declared done before its gather and copies have run: waits would
// return early, parked blocks would be released early and a later swap-in would skip its
// conflict wait.  This test builds a pool object by hand (no device, no HIP call: the event
// pool is pre-filled with stand-in handles and the completion test is replaced by one that
// reports "complete" for everything, which is what the runtime does for such events) and
// checks that polling leaves an op alone until it is marked issued.
#include <stdio.h>

#include "../../paper_2411_18424_amd/csrc/kv_pool.hpp"

static int g_fail = 0;
#define EXPECT(c)                                                   \
  do {                                                              \
    if (!(c)) {                                                     \
      fprintf(stderr, "FAIL %s:%d: %s\n", __FILE__, __LINE__, #c);  \
      ++g_fail;                                                     \
    }                                                               \
  } while (0)

static hipError_t always_complete(hipEvent_t) { return hipSuccess; }

int main() {
  kv_pool p;
  p.plan = false;
  p.N = 16;
  p.alloc.init(p.N);
  p.reader_seq.assign(16, 0);
  p.writer_seq.assign(16, 0);
  p.event_query = always_complete;
  for (uintptr_t i = 1; i <= 32; ++i) p.event_pool.push_back((hipEvent_t)(i << 8));  // never dereferenced

  // a swap-out being enqueued
  kvi::OpRef out;
  EXPECT(kvi::new_op(&p, true, &out) == KV_OK);
  EXPECT(out->seq == 1 && !out->issued);
  // blocks it reads are freed meanwhile: they must stay parked
  int32_t ids[3] = {2, 3, 4};
  int32_t got = 0;
  {
    std::vector<int32_t> v;
    got = p.alloc.alloc(16, &v);
    EXPECT(got == 1 && v.size() == 16);
  }
  for (int32_t b : ids) p.reader_seq[(size_t)b] = out->seq;
  p.alloc.free_ids(ids, 3, p.reader_seq, p.pack_done_seq, p.writer_seq, p.scat_done_seq);
  EXPECT(p.alloc.n_draining() == 3 && p.alloc.n_free() == 0);

  kvi::reap(&p);
  EXPECT(!out->packed_done && !out->all_done);
  EXPECT(p.pack_done_seq == 0);
  EXPECT(p.ops_out.size() == 1);
  EXPECT(out->packed != nullptr && out->done != nullptr);  // events not recycled under it
  EXPECT(p.alloc.n_draining() == 3);                        // blocks not released early

  // a swap-in being enqueued behaves the same
  kvi::OpRef in;
  EXPECT(kvi::new_op(&p, false, &in) == KV_OK);
  kvi::reap(&p);
  EXPECT(!in->all_done && p.scat_done_seq == 0 && p.ops_in.size() == 1);

  // an issued op behind an unissued one is not overtaken (ops finish in issue order)
  kvi::OpRef out2;
  EXPECT(kvi::new_op(&p, true, &out2) == KV_OK);
  out2->issued = out2->packed_recorded = true;
  kvi::reap(&p);
  EXPECT(!out2->packed_done && p.pack_done_seq == 0 && p.ops_out.size() == 2);

  // a swap-out whose copies are held back: its gathers are enqueued and their event recorded, its
  // completion event is not.  The gather counts as finished (the blocks it read are released, and
  // so is the gather of the op behind it), completion does not, and no event is recycled.
  out->packed_recorded = true;
  kvi::reap(&p);
  EXPECT(out->packed_done && !out->all_done && out2->packed_done && !out2->all_done);
  EXPECT(p.pack_done_seq == 2 && p.ops_out.size() == 2);
  EXPECT(out->packed != nullptr && out->done != nullptr);
  EXPECT(p.alloc.n_draining() == 0 && p.alloc.n_free() == 3);

  // once issued, everything is harvested in order
  out->issued = true;
  in->issued = true;
  kvi::reap(&p);
  EXPECT(out->all_done && out2->all_done && in->all_done);
  EXPECT(p.pack_done_seq == 2 && p.scat_done_seq == 1);
  EXPECT(p.ops_out.empty() && p.ops_in.empty());
  EXPECT(out->packed == nullptr && out->done == nullptr);
  EXPECT(p.alloc.n_draining() == 0 && p.alloc.n_free() == 3);

  // room of the out ring beside swap-outs whose copies have not been enqueued yet: the bytes from
  // the ring head forward to the oldest such region, less one piece held in reserve for a skipped tail
  {
    p.R = 10;
    kvi::ByteRing& r = p.ring_out;
    r.cap = 1000;
    r.piece_blocks = 5;  // pieces of 50 bytes
    r.head = 0;
    EXPECT(kvi::out_ring_room(&p) == 950);  // nothing held back
    auto region = [](int64_t off, int64_t len, bool recorded) {
      kvi::Region g;
      g.off = off;
      g.len = len;
      g.recorded = recorded;
      return g;
    };
    r.live = {region(100, 200, true), region(300, 100, false), region(400, 100, false)};
    r.head = 500;
    EXPECT(kvi::out_ring_room(&p) == 500 + 300 - 50);  // to the end, around, up to offset 300
    r.live = {region(700, 100, false), region(800, 100, true)};
    r.head = 900;  // (a recorded region behind an open one cannot arise; the oldest open one decides anyway)
    EXPECT(kvi::out_ring_room(&p) == 100 + 700 - 50);
    r.live = {region(600, 300, false)};
    r.head = 100;  // wrapped: the open region lies ahead of the head
    EXPECT(kvi::out_ring_room(&p) == 500 - 50);
    r.live = {region(120, 900 - 120, false)};
    r.head = 100;  // nearly full
    EXPECT(kvi::out_ring_room(&p) == 0);
    r.live.clear();
    r.head = 0;
  }

  p.event_pool.clear();  // stand-in handles: nothing to destroy
  printf("reap_unissued: %d failures\n", g_fail);
  return g_fail ? 1 : 0;
}
