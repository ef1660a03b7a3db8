// Internal declarations shared by the translation units of the KV-swap library: the pool
// object and its parts, and the functions that cross file boundaries.  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <chrono>
#include <condition_variable>
#include <deque>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/kvswap.h"
#include "kv_alloc.hpp"
#include "kv_kernels.h"


struct kv_pool;

namespace kvi {

extern thread_local std::string g_err;
int32_t fail(int32_t code, const char* fmt, ...);

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
  bool issued = false;          // every event of the op has been recorded (or the enqueue has failed);
                                // until then completion polling must not look at them: a query of an
                                // event that was never recorded, or was recycled, reports success
  bool packed_recorded = false; // `packed` has been recorded (a swap-out whose copies are held back
                                // has its gathers enqueued and this set long before `issued`)
  bool deferred = false;        // the copy thread finishes the enqueue and sets `issued`
  std::vector<hipEvent_t> aux;  // hand-off events of this op, recycled when it is done
  std::vector<hipEvent_t> timed;  // begin / end events attached to the pack launches of a large op (see launch_pack)
  std::vector<hipEvent_t> layer_ev;  // layer-wise swap-in: one per step of layer_step layers (null
                                     // entries in a plan-only pool); recycled when the op is done
  int32_t layer_step = 0;
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

// One host<->device copy of a swap: `rows` rows of `width` bytes, `pitch` bytes apart on the host
// side and packed in staging (rows == 1: a plain contiguous copy).  Offsets are bytes into the
// arena and into the staging slot.
struct CopyDesc {
  int64_t host_off, slot_off, width, rows, pitch;
};
// KV_FLAG_SECOND_LANE: which pieces of a held-back swap-out travel as plain copies on two streams
constexpr int64_t KV_SECOND_LANE_MIN_COPIES = 8;
constexpr int64_t KV_SECOND_LANE_MIN_AVG_BYTES = 1ll << 20;     // average copy of 1 MiB ... 8 MiB: the sizes measured
constexpr int64_t KV_SECOND_LANE_MAX_AVG_BYTES = 8ll << 20;
constexpr int64_t KV_SECOND_LANE_MAX_PIECE_BYTES = 512ll << 20;  // bounds what a swap-in that arrives meanwhile queues behind
constexpr int64_t KV_MAX_COPY_PITCH = 1ll << 30;      // largest host pitch of a 2-D copy (measured up to here)
constexpr int64_t KV_MAX_STRIDED_WIDTH = 16ll << 20;  // widest row of a 2-D copy (measured up to here)

// A swap-out whose copies are held back until its gathers have finished (the default for swap-outs of defer_min_bytes or more):
// the pieces already gathered into the staging ring, each with the event recorded behind its
// gathers.  The pool's copy thread waits for each event on the host and only then hands the
// piece's copies to the runtime.
struct DeferredPiece {
  int64_t first, count, off;  // moves [first, first + count) lie at ring offset off
  hipEvent_t ready;
};
struct DeferredOut {
  OpRef op;
  std::vector<Move> mv;
  std::vector<DeferredPiece> pieces;
};

struct ProfRec {
  int32_t kind;
  int64_t bytes;
  hipEvent_t start, stop;
};

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

// One request of a (possibly batched) swap-in, after validation.
struct InItem {
  int64_t req;
  const int32_t* table;
  int32_t n;
  const uint8_t* resident;  // null = move everything
};

}  // namespace kvi

struct kv_pool {
  kv_pool_config_t cfg{};
  bool plan = false, profile = false, order_compute = false, four_streams = false;
  int64_t N = 0, C = 0, R = 0;
  int32_t P = 0;
  char* gpu = nullptr;
  char* host = nullptr;      // pinned arena
  char* host_dev = nullptr;  // the arena as the device addresses it
  bool mapped_in = false;
  bool mapped_out = false;          // swap-outs of at most mapped_out_max blocks store to the host directly
  int64_t mapped_out_max = 0;       // 0 = no limit
  bool host_evict = false;
  uint64_t use_clock = 0;
  int mapped_grid = 64;
  int64_t arena_blocks = 0;
  bool own_staging = false;
  char* staging = nullptr;
  char* static_staging = nullptr;  // this device's address of the library's file-scope staging array
  kvi::ByteRing ring_out, ring_in;
  hipStream_t s_pack = nullptr, s_d2h = nullptr, s_h2d = nullptr, s_scat = nullptr;
  hipStream_t compute = nullptr;
  hipEvent_t ev_compute = nullptr;
  int unroll = 0, grid = 0, variant = 0;
  int64_t launch_blocks = KV_MAX_LAUNCH_BLOCKS;  // most blocks one pack launch carries
  int64_t copy_chunk = 0;
  bool defer_copies = true;   // off with KV_FLAG_NO_DEFER_COPIES
  int64_t defer_min = 0;      // smallest swap-out (bytes) whose copies are held back
  bool second_lane = false;   // KV_FLAG_SECOND_LANE
  bool launch_events = true;  // off with KV_FLAG_NO_LAUNCH_EVENTS
  int device = 0;             // the device that was current when the pool was created
  bool strided_copies = true;  // equal runs a constant stride apart go out as rows of one 2-D copy
  int64_t slack = 32;

  std::mutex mu;
  std::unordered_map<int64_t, kvi::Req> reqs;
  kv::RunSet arena;
  kv::BlockGroupAllocator alloc;
  kv::BlockGroupManager groups;
  std::vector<uint64_t> reader_seq, writer_seq;  // per physical block
  std::vector<uint32_t> stamp;                   // duplicate detection
  uint32_t epoch = 0;
  std::vector<uint32_t> free_stamp;
  uint32_t free_epoch = 0;

  std::deque<kvi::OpRef> ops_out, ops_in;
  uint64_t out_seq = 0, in_seq = 0;
  uint64_t pack_done_seq = 0, scat_done_seq = 0;
  std::vector<hipEvent_t> event_pool;   // timing disabled
  std::vector<hipEvent_t> timing_pool;  // timing enabled
  std::vector<kvi::ProfRec> prof;
  kv_stats_t st{};
  // swap-outs whose copies are held back, in issue order, and the thread that releases them
  std::deque<kvi::DeferredOut> jobs;
  int deferred_pending = 0;  // jobs queued or in the copy thread's hands
  std::condition_variable_any cv_job, cv_issued;  // waited for with `mu` held
  std::thread copy_thread;
  bool copy_thread_stop = false;
  int32_t copy_thread_rc = 0;  // first error of the copy thread, reported by the calls that wait for its work
  std::string copy_thread_err;
  // completion test of an event (hipEventQuery); a host-only unit test substitutes its own
  hipError_t (*event_query)(hipEvent_t) = hipEventQuery;
};

namespace kvi {

// kv_engine.cpp: events, completion polling, staging rings, kernel launches and copies
int32_t get_event(kv_pool* p, hipEvent_t* ev);
int32_t get_timing_event(kv_pool* p, hipEvent_t* ev);
void put_event(kv_pool* p, hipEvent_t ev);
void reap(kv_pool* p);
Op* find_op(std::deque<OpRef>& dq, uint64_t seq);
int32_t host_wait_op(kv_pool* p, const OpRef& op);
int32_t wait_issued(kv_pool* p, const OpRef& op);  // lock held; returns once the op's events are all recorded
int32_t wait_all_issued(kv_pool* p);               // the same for every swap-out handed to the copy thread
int64_t out_ring_room(kv_pool* p);                 // bytes a swap-out can claim without reaching a held-back one's regions
void stop_copy_thread(kv_pool* p, std::unique_lock<std::mutex>& lk);
int32_t new_op(kv_pool* p, bool is_out, OpRef* out);
void order_for_strided_copies(kv_pool* p, std::vector<Move>& mv);
void plan_copies(const Move* mv, int64_t m, int64_t R, int64_t copy_chunk, bool strided, std::vector<CopyDesc>* out);
int32_t enqueue_out(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                    const OpRef& op);
int32_t enqueue_in(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre_copy,
                   const std::vector<hipEvent_t>& pre_scat, const OpRef& op);
int32_t enqueue_in_layers(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre_copy,
                          const std::vector<hipEvent_t>& pre_scat, const OpRef& op, int32_t step);
int32_t enqueue_direct(kv_pool* p, bool to_host, const std::vector<Move>& mv,
                       const std::vector<hipEvent_t>& pre, const OpRef& op, bool per_block);
int32_t enqueue_out_mapped(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                           const OpRef& op);
int32_t enqueue_in_mapped(kv_pool* p, const std::vector<Move>& mv, const std::vector<hipEvent_t>& pre,
                          const OpRef& op, int32_t layer_step = 0);

// kv_reuse.cpp: validation, host arena and images, moved-set selection (the reuse map)
void arena_give(kv_pool* p, const std::vector<Extent>& ext);
int32_t do_swap_out(kv_pool* p, std::vector<OutItem>& items, int32_t* out_n_moved, int direct = 0);
int32_t do_swap_in(kv_pool* p, std::vector<InItem>& items, int32_t* out_n_moved, int direct = 0,
                   int32_t layer_step = 0);

}  // namespace kvi
