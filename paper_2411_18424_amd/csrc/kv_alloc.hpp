// Block-group allocator and host-arena allocator (host-side bookkeeping, no HIP).
//
// Block groups follow FastSwitch (arXiv 2411.18424) Section 3.1: KV blocks are handed out
// in contiguous runs ("block groups") in the manner of a buddy allocator - all blocks start
// merged into one free group, a group is split on demand, adjacent free groups merge - so
// that a request's blocks sit in few large extents.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <map>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

namespace kv {

// Free runs of a 1-D id space, indexed by address (merge) and by size (fit).
class RunSet {
 public:
  void clear() {
    by_addr_.clear();
    by_size_.clear();
    total_ = 0;
  }
  int64_t total() const { return total_; }
  int64_t largest() const { return by_size_.empty() ? 0 : by_size_.rbegin()->first; }
  size_t n_runs() const { return by_addr_.size(); }

  // Insert [start, start+len), merging with free neighbours.
  void insert(int64_t start, int64_t len) {
    if (len <= 0) return;
    total_ += len;
    auto next = by_addr_.lower_bound(start);
    if (next != by_addr_.begin()) {
      auto prev = std::prev(next);
      if (prev->first + prev->second == start) {
        start = prev->first;
        len += prev->second;
        by_size_.erase({prev->second, prev->first});
        by_addr_.erase(prev);
      }
    }
    if (next != by_addr_.end() && start + len == next->first) {
      len += next->second;
      by_size_.erase({next->second, next->first});
      by_addr_.erase(next);
    }
    by_addr_[start] = len;
    by_size_.insert({len, start});
  }

  // Best fit: the smallest run with len >= n, lowest address on ties.  Takes its low end.
  bool take_best_fit(int64_t n, int64_t* start) {
    auto it = by_size_.lower_bound({n, INT64_MIN});
    if (it == by_size_.end()) return false;
    carve(it->second, it->first, n);
    *start = last_start_;
    return true;
  }

  // As take_best_fit(n), but only among runs of at least min_len blocks.
  bool take_best_fit_at_least(int64_t n, int64_t min_len, int64_t* start) {
    auto it = by_size_.lower_bound({std::max(n, min_len), INT64_MIN});
    if (it == by_size_.end()) return false;
    carve(it->second, it->first, n);
    *start = last_start_;
    return true;
  }

  // Takes the low end (up to n) of the largest run; returns the length taken.
  int64_t take_from_largest(int64_t n, int64_t* start) {
    if (by_size_.empty()) return 0;
    auto it = std::prev(by_size_.end());
    // lowest address among the largest runs
    auto lo = by_size_.lower_bound({it->first, INT64_MIN});
    int64_t take = std::min<int64_t>(n, lo->first);
    carve(lo->second, lo->first, take);
    *start = last_start_;
    return take;
  }

  // Takes the high end (n records) of the largest run, if it is that long.
  bool take_top_of_largest(int64_t n, int64_t* start) {
    if (by_size_.empty()) return false;
    auto it = std::prev(by_size_.end());
    auto lo = by_size_.lower_bound({it->first, INT64_MIN});
    if (lo->first < n) return false;
    const int64_t s = lo->second + lo->first - n;
    if (!take_exact(s, n)) return false;
    *start = s;
    return true;
  }

  // Takes [start, start+len) if it is entirely free (used to extend a region in place).
  bool take_exact(int64_t start, int64_t len) {
    auto it = by_addr_.upper_bound(start);
    if (it == by_addr_.begin()) return false;
    --it;
    int64_t rs = it->first, rl = it->second;
    if (start < rs || start + len > rs + rl) return false;
    by_size_.erase({rl, rs});
    by_addr_.erase(it);
    total_ -= rl;
    insert(rs, start - rs);
    insert(start + len, rs + rl - (start + len));
    return true;
  }

  const std::map<int64_t, int64_t>& runs() const { return by_addr_; }

 private:
  void carve(int64_t start, int64_t len, int64_t n) {
    by_size_.erase({len, start});
    by_addr_.erase(start);
    total_ -= len;
    last_start_ = start;
    if (len > n) insert(start + n, len - n);
  }
  std::map<int64_t, int64_t> by_addr_;           // start -> len
  std::set<std::pair<int64_t, int64_t>> by_size_;  // (len, start)
  int64_t total_ = 0;
  int64_t last_start_ = 0;
};

// Allocator of GPU KV blocks in contiguous runs.
class BlockGroupAllocator {
 public:
  enum State : uint8_t { FREE = 0, USED = 1, DRAINING = 2 };

  void init(int64_t n_blocks) {
    n_ = n_blocks;
    state_.assign((size_t)n_blocks, FREE);
    free_.clear();
    free_.insert(0, n_blocks);
    draining_.clear();
    n_draining_ = 0;
  }
  int64_t n_free() const { return free_.total(); }
  int64_t n_draining() const { return n_draining_; }
  int64_t largest_run() const { return free_.largest(); }

  // Allocates n ids into out (which must be empty), fewest runs first: the best-fitting free
  // run if one holds the rest, else the largest run, repeatedly.  A request that has to be
  // split therefore uses the longest free runs first; its last piece (the remainder, which may
  // be short) is carved from the best-fitting run of at least min_run blocks when there is
  // one, so that free runs shorter than min_run are touched only when every longer run is used
  // up - the short fragments stay for requests that are short themselves.  A request that fits
  // one free run takes the best-fitting one whatever min_run says.  Caller has checked
  // n <= n_free().  Returns the number of maximal runs of consecutive ids in out.
  int32_t alloc(int64_t n, std::vector<int32_t>* out, int64_t min_run = 1) {
    int64_t start;
    bool split = false;
    while (n > 0) {
      int64_t got;
      if (split && n < min_run && free_.take_best_fit_at_least(n, min_run, &start)) {
        got = n;
      } else if (free_.take_best_fit(n, &start)) {
        got = n;
      } else {
        got = free_.take_from_largest(n, &start);
        split = true;
      }
      for (int64_t i = 0; i < got; ++i) {
        state_[(size_t)(start + i)] = USED;
        out->push_back((int32_t)(start + i));
      }
      n -= got;
    }
    return count_runs(*out);
  }

  // One contiguous run of up to `want` blocks: the best-fitting free run if one holds `want`,
  // else the largest free run (shorter).  Returns the length taken (0 if nothing is free).
  int64_t alloc_run(int64_t want, int64_t* start) {
    if (want <= 0) return 0;
    int64_t got = want;
    if (!free_.take_best_fit(want, start)) got = free_.take_from_largest(want, start);
    for (int64_t i = 0; i < got; ++i) state_[(size_t)(*start + i)] = USED;
    return got;
  }

  // Extends a used run in place: takes [start, start+len) if it is entirely free.
  bool alloc_exact(int64_t start, int64_t len) {
    if (len <= 0 || start < 0 || start + len > n_) return false;
    if (!free_.take_exact(start, len)) return false;
    for (int64_t i = 0; i < len; ++i) state_[(size_t)(start + i)] = USED;
    return true;
  }

  // True if every id is in range, USED and named once.  scratch is a caller-kept stamp array.
  bool can_free(const int32_t* ids, int32_t n, std::vector<uint32_t>* stamp, uint32_t* epoch) const {
    if ((int64_t)stamp->size() != n_) stamp->assign((size_t)n_, 0);
    ++*epoch;
    for (int32_t i = 0; i < n; ++i) {
      int64_t b = ids[i];
      if (b < 0 || b >= n_ || state_[(size_t)b] != USED) return false;
      if ((*stamp)[(size_t)b] == *epoch) return false;
      (*stamp)[(size_t)b] = *epoch;
    }
    return true;
  }

  // Frees ids.  A block that an unfinished gather still reads (reader_seq[b] > out_done) or an
  // unfinished scatter still writes (writer_seq[b] > in_done) is parked, and released by
  // reap() once both have finished; it is never handed out before.
  void free_ids(const int32_t* ids, int32_t n, const std::vector<uint64_t>& reader_seq, uint64_t out_done,
                const std::vector<uint64_t>& writer_seq, uint64_t in_done) {
    std::vector<int32_t> v(ids, ids + n);
    std::sort(v.begin(), v.end());
    auto busy = [&](int32_t b) {
      return reader_seq[(size_t)b] > out_done || writer_seq[(size_t)b] > in_done;
    };
    size_t i = 0;
    while (i < v.size()) {
      size_t j = i;
      const bool parked = busy(v[i]);
      uint64_t max_out = reader_seq[(size_t)v[i]], max_in = writer_seq[(size_t)v[i]];
      while (j + 1 < v.size() && v[j + 1] == v[j] + 1 && busy(v[j + 1]) == parked) {
        ++j;
        max_out = std::max(max_out, reader_seq[(size_t)v[j]]);
        max_in = std::max(max_in, writer_seq[(size_t)v[j]]);
      }
      int64_t start = v[i], len = (int64_t)(j - i + 1);
      if (parked) {
        for (int64_t k = 0; k < len; ++k) state_[(size_t)(start + k)] = DRAINING;
        draining_.push_back({max_out, max_in, start, len});
        n_draining_ += len;
      } else {
        for (int64_t k = 0; k < len; ++k) state_[(size_t)(start + k)] = FREE;
        free_.insert(start, len);
      }
      i = j + 1;
    }
  }

  // Releases parked runs whose gather (sequence <= out_done) and scatter (<= in_done) have
  // both finished.
  void reap(uint64_t out_done, uint64_t in_done) {
    size_t w = 0;
    for (size_t i = 0; i < draining_.size(); ++i) {
      Parked& d = draining_[i];
      if (d.out_seq <= out_done && d.in_seq <= in_done) {
        for (int64_t k = 0; k < d.len; ++k) state_[(size_t)(d.start + k)] = FREE;
        free_.insert(d.start, d.len);
        n_draining_ -= d.len;
      } else {
        draining_[w++] = d;
      }
    }
    draining_.resize(w);
  }

  // The gather and the scatter whose completion would release at least `need` parked blocks,
  // oldest work first (*out_seq / *in_seq: wait for ops up to these; 0 = none of that kind).
  // False if even all parked blocks are not enough.
  bool seqs_to_release(int64_t need, uint64_t* out_seq, uint64_t* in_seq) const {
    std::vector<const Parked*> v;
    for (const Parked& d : draining_) v.push_back(&d);
    std::sort(v.begin(), v.end(), [](const Parked* a, const Parked* b) {
      return a->out_seq + a->in_seq < b->out_seq + b->in_seq;
    });
    *out_seq = *in_seq = 0;
    int64_t got = 0;
    for (const Parked* d : v) {
      *out_seq = std::max(*out_seq, d->out_seq);
      *in_seq = std::max(*in_seq, d->in_seq);
      got += d->len;
      if (got >= need) return true;
    }
    return false;
  }

  uint8_t state(int64_t b) const { return state_[(size_t)b]; }

 private:
  struct Parked {
    uint64_t out_seq, in_seq;  // last gather reading / last scatter writing the run
    int64_t start, len;
  };
  static int32_t count_runs(const std::vector<int32_t>& ids) {
    if (ids.empty()) return 0;
    int32_t r = 1;
    for (size_t i = 1; i < ids.size(); ++i)
      if (ids[i] != ids[i - 1] + 1) ++r;
    return r;
  }
  int64_t n_ = 0;
  std::vector<uint8_t> state_;
  RunSet free_;
  std::vector<Parked> draining_;
  int64_t n_draining_ = 0;
};

// Dynamic Block Group Manager (Section 3.1): requests own block groups (contiguous runs); the
// newest group of a request is its active group, whose unused tail the request grows into
// and from which other requests may be served when the free groups run out.
class BlockGroupManager {
 public:
  struct Group {
    int64_t start, len, used;  // blocks [start, start+used) hold KV, the rest is reserved tail
  };
  struct Stats {
    int64_t n_requests = 0, n_groups = 0, used_blocks = 0, tail_blocks = 0;
    int64_t steals = 0, opened = 0, appended_groups = 0, grown_in_place = 0;
  };

  void configure(BlockGroupAllocator* a, int64_t first_group, uint64_t seed) {
    alloc_ = a;
    first_group_ = first_group > 0 ? first_group : 64;
    rng_ = seed ? seed : 0x9E3779B97F4A7C15ull;
  }
  int64_t first_group() const { return first_group_; }
  bool has(int64_t req) const { return owners_.count(req) != 0; }

  // Blocks the manager could still hand to `req`: free blocks plus the tails of other
  // requests' active groups.
  int64_t obtainable(int64_t req) const {
    int64_t n = alloc_->n_free();
    for (const auto& kv : owners_)
      if (kv.first != req && !kv.second.empty()) n += kv.second.back().len - kv.second.back().used;
    auto f = owners_.find(req);
    if (f != owners_.end() && !f->second.empty()) n += f->second.back().len - f->second.back().used;
    return n;
  }

  // Gives `req` n more blocks (appended to out): from its active group's tail, then by
  // growing that group in place, then from new groups of the expected size (first_group,
  // shrunk to what is free), then from the tail of a randomly chosen other request's active
  // group.  Caller has checked n <= obtainable(req).
  void append(int64_t req, int64_t n, int64_t reserve_tail, std::vector<int32_t>* out) {
    std::vector<Group>& gs = owners_[req];
    while (n > 0) {
      if (!gs.empty() && gs.back().used < gs.back().len) {
        Group& g = gs.back();
        int64_t k = std::min(n, g.len - g.used);
        for (int64_t i = 0; i < k; ++i) out->push_back((int32_t)(g.start + g.used + i));
        g.used += k;
        n -= k;
        continue;
      }
      if (!gs.empty()) {  // grow the active group where it stands
        Group& g = gs.back();
        int64_t want = std::max(n, std::min(first_group_, reserve_tail + n));
        while (want >= n && want > 0 && !alloc_->alloc_exact(g.start + g.len, want)) want = want > n ? n : 0;
        if (want > 0) {
          g.len += want;
          ++st_.grown_in_place;
          continue;
        }
      }
      int64_t start, want = std::max(n + reserve_tail, gs.empty() ? std::max(n, first_group_) : first_group_);
      int64_t got = alloc_->alloc_run(want, &start);
      if (got > 0) {
        gs.push_back({start, got, 0});
        gs.size() == 1 ? ++st_.opened : ++st_.appended_groups;
        continue;
      }
      if (!steal(req, n, &gs)) break;  // nothing obtainable (caller checked, so not reached)
    }
  }

  // The request's block table: used blocks of its groups in order.
  void table(int64_t req, std::vector<int32_t>* out) const {
    auto f = owners_.find(req);
    if (f == owners_.end()) return;
    for (const Group& g : f->second)
      for (int64_t i = 0; i < g.used; ++i) out->push_back((int32_t)(g.start + i));
  }

  // All blocks of the request, tails included (for release).
  void all_blocks(int64_t req, std::vector<int32_t>* out) const {
    auto f = owners_.find(req);
    if (f == owners_.end()) return;
    for (const Group& g : f->second)
      for (int64_t i = 0; i < g.len; ++i) out->push_back((int32_t)(g.start + i));
  }
  void forget(int64_t req) { owners_.erase(req); }

  Stats stats() const {
    Stats s = st_;
    s.n_requests = (int64_t)owners_.size();
    for (const auto& kv : owners_)
      for (const Group& g : kv.second) {
        if (g.used > 0) ++s.n_groups;
        s.used_blocks += g.used;
        s.tail_blocks += g.len - g.used;
      }
    return s;
  }

 private:
  uint64_t next_random() {  // splitmix64
    uint64_t z = (rng_ += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }

  // No free group is left: split the unused tail of a randomly selected other request's
  // active group - all of it if it is no longer than the need, else the need or half of it,
  // whichever is more - and give the split-off end to `req` as a new group.
  bool steal(int64_t req, int64_t need, std::vector<Group>* gs) {
    std::vector<int64_t> victims;
    for (const auto& kv : owners_)
      if (kv.first != req && !kv.second.empty() && kv.second.back().len > kv.second.back().used)
        victims.push_back(kv.first);
    if (victims.empty()) return false;
    std::sort(victims.begin(), victims.end());  // map order is not deterministic
    Group& v = owners_[victims[(size_t)(next_random() % victims.size())]].back();
    const int64_t tail = v.len - v.used;
    const int64_t k = tail <= need ? tail : std::max(need, tail / 2);
    v.len -= k;
    gs->push_back({v.start + v.len, k, 0});
    ++st_.steals;
    return true;
  }

  BlockGroupAllocator* alloc_ = nullptr;
  int64_t first_group_ = 64;
  uint64_t rng_ = 0;
  std::unordered_map<int64_t, std::vector<Group>> owners_;
  Stats st_;
};

}  // namespace kv
