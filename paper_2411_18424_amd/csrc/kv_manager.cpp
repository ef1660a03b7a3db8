// Swap manager: asynchronous dispatch of swaps (FastSwitch, arXiv 2411.18424, Section 3.2,
// Algorithm 1).
//
// The paper moves the dispatch of swap copies off the scheduler's thread onto a C++ thread
// pool, records progress with events taken from a pool, lets the scheduler poll for finished
// swap-ins at the start of every iteration (step 1), and decides per iteration whether
// pending swap-ins proceed asynchronously or the scheduler stalls for them (step 4), from a
// window of recent swap statistics (r_info).
//
// Here a swap is a handful of runtime calls (one pack launch per ~1.75 GiB, one copy per run),
// not one call per block group, so one dispatcher thread is enough; it also keeps tasks in
// submission order, which the pool's conflict detection relies on (a swap-in into blocks a
// queued swap-out is about to read must be dispatched after it).  submit() copies the table
// and returns in about a microsecond; the dispatcher calls the pool's entry points; poll()
// reports tasks whose device work has finished.

#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/kvswap.h"

namespace {

using Clock = std::chrono::steady_clock;

struct Task {
  uint64_t ticket = 0;
  int32_t kind = 0;
  int64_t req = 0;
  std::vector<int32_t> table;
  std::vector<uint8_t> mask;
  bool free_blocks = false;  // swap-outs: give the table's blocks back to the allocator once dispatched
  Clock::time_point t_submit;
};

struct Flight {  // dispatched, device work possibly still running
  uint64_t ticket;
  int64_t req;
  int32_t status;
};

struct Recent {  // one entry of the r_info window
  int32_t kind;
  int64_t blocks;
  double dispatch_us;
};

}  // namespace

struct kv_manager {
  kv_pool_t* pool = nullptr;
  kv_manager_config_t cfg{};
  int64_t record_bytes = 0;

  std::mutex mu;
  std::condition_variable cv_work, cv_done;
  std::deque<Task> queue;
  std::deque<Flight> flights;                        // in dispatch order
  std::unordered_map<uint64_t, int32_t> finished;    // ticket -> status, not yet reported
  std::deque<uint64_t> finished_order;
  std::deque<Recent> window;
  uint64_t next_ticket = 1;
  uint64_t dispatched_upto = 0;  // every ticket <= this has been dispatched
  bool stop = false;
  std::thread worker;
  kv_manager_stats_t st{};

  // Algorithm 1's queues, kept by kv_manager_iterate: where each request is, and the
  // swap-ins / swap-outs whose outcome has not been booked yet.
  enum Where : uint8_t { RUNNING = 0, SWAPPED = 1, ONGOING_SWAP_IN = 2 };
  struct Pending {
    int64_t req;
    uint64_t ticket;
  };
  std::unordered_map<int64_t, uint8_t> where;
  std::vector<Pending> ongoing_swap_in, pending_out;
  std::vector<std::pair<int64_t, int32_t>> failures;  // (request, status), reported by the next iterate
  kv_iteration_stats_t it_st{};
};

namespace {

int32_t dispatch(kv_manager* m, Task& t) {
  const int32_t n = (int32_t)t.table.size();
  const int32_t* tab = n ? t.table.data() : nullptr;
  const uint8_t* mask = t.mask.empty() ? nullptr : t.mask.data();
  int32_t rc = KV_EINVAL;
  switch (t.kind) {
    case KV_TASK_SWAP_OUT:
      rc = swap_out(m->pool, t.req, tab, n);
      break;
    case KV_TASK_SWAP_IN:
      return swap_in(m->pool, t.req, tab, n);
    case KV_TASK_SWAP_OUT_DELTA:
      rc = swap_out_delta(m->pool, t.req, tab, n, mask, nullptr);
      break;
    case KV_TASK_SWAP_IN_DELTA:
      return swap_in_delta(m->pool, t.req, tab, n, mask, nullptr);
  }
  // preemption gives the victim's blocks up: only now that the gather is enqueued does the
  // allocator know to hold them back until it has read them
  if (rc == KV_OK && t.free_blocks && n > 0) rc = free_block_group(m->pool, t.req, tab, n);
  return rc;
}

// Moves flights whose device work has finished to the finished list.  Lock held.
void harvest(kv_manager* m) {
  while (!m->flights.empty()) {
    Flight& f = m->flights.front();
    int32_t done = 1;
    if (f.status == KV_OK && kv_query(m->pool, f.req, &done) != KV_OK) done = 1;
    if (!done) break;  // ops of one request finish in order; later flights are polled below
    m->finished[f.ticket] = f.status;
    m->finished_order.push_back(f.ticket);
    m->flights.pop_front();
  }
  // flights behind an unfinished one may belong to other requests and be done already
  // (kv_query speaks for a request's last dispatched op; its ops finish in order)
  for (size_t i = 1; i < m->flights.size();) {
    Flight& f = m->flights[i];
    int32_t done = 1;
    if (f.status == KV_OK && kv_query(m->pool, f.req, &done) != KV_OK) done = 1;
    if (done) {
      m->finished[f.ticket] = f.status;
      m->finished_order.push_back(f.ticket);
      m->flights.erase(m->flights.begin() + (long)i);
    } else {
      ++i;
    }
  }
}

void worker_loop(kv_manager* m) {
  std::unique_lock<std::mutex> lk(m->mu);
  for (;;) {
    m->cv_work.wait(lk, [&] { return m->stop || !m->queue.empty(); });
    if (m->queue.empty()) {
      if (m->stop) return;
      continue;
    }
    Task t = std::move(m->queue.front());
    m->queue.pop_front();
    lk.unlock();
    const auto t0 = Clock::now();
    const int32_t status = dispatch(m, t);
    const auto t1 = Clock::now();
    lk.lock();
    const double us = std::chrono::duration<double, std::micro>(t1 - t0).count();
    const double wait_us = std::chrono::duration<double, std::micro>(t0 - t.t_submit).count();
    m->st.dispatched++;
    m->st.dispatch_us_sum += us;
    m->st.queue_wait_us_sum += wait_us;
    if (status != KV_OK) m->st.failed++;
    m->flights.push_back({t.ticket, t.req, status});
    m->dispatched_upto = t.ticket;
    m->window.push_back({t.kind, (int64_t)t.table.size(), us});
    while ((int32_t)m->window.size() > m->cfg.window) m->window.pop_front();
    m->cv_done.notify_all();
  }
}

}  // namespace

extern "C" {

int32_t kv_manager_create(kv_pool_t* pool, const kv_manager_config_t* cfg, kv_manager_t** out) {
  if (!pool || !out) return KV_EINVAL;
  int64_t record_bytes = 0;
  if (kv_record_bytes(pool, &record_bytes) != KV_OK || record_bytes <= 0) return KV_EINVAL;
  kv_manager* m = new kv_manager();
  m->pool = pool;
  if (cfg) m->cfg = *cfg;
  if (m->cfg.window <= 0) m->cfg.window = 64;
  if (m->cfg.link_gbps <= 0) m->cfg.link_gbps = 55.0;
  if (m->cfg.sync_below_ms <= 0) m->cfg.sync_below_ms = 0.5;
  m->record_bytes = record_bytes;
  m->worker = std::thread(worker_loop, m);
  *out = m;
  return KV_OK;
}

int32_t kv_manager_destroy(kv_manager_t* m) {
  if (!m) return KV_EINVAL;
  {
    std::lock_guard<std::mutex> g(m->mu);
    m->stop = true;
  }
  m->cv_work.notify_all();
  m->worker.join();  // the queue is drained before the worker returns
  kv_wait_all(m->pool);
  delete m;
  return KV_OK;
}

static int32_t submit_task(kv_manager_t* m, int32_t kind, int64_t req, const int32_t* table, int32_t n,
                           const uint8_t* mask, uint64_t* ticket, bool free_blocks);

int32_t kv_manager_submit(kv_manager_t* m, int32_t kind, int64_t req, const int32_t* table, int32_t n,
                          const uint8_t* mask, uint64_t* ticket) {
  return submit_task(m, kind, req, table, n, mask, ticket, false);
}

static int32_t submit_task(kv_manager_t* m, int32_t kind, int64_t req, const int32_t* table, int32_t n,
                           const uint8_t* mask, uint64_t* ticket, bool free_blocks) {
  if (!m || n < 0 || (n > 0 && !table) || kind < KV_TASK_SWAP_OUT || kind > KV_TASK_SWAP_IN_DELTA)
    return KV_EINVAL;
  if ((kind == KV_TASK_SWAP_OUT_DELTA || kind == KV_TASK_SWAP_IN_DELTA) && n > 0 && !mask) return KV_EINVAL;
  Task t;
  t.kind = kind;
  t.req = req;
  t.table.assign(table, table + n);
  if (mask && (kind == KV_TASK_SWAP_OUT_DELTA || kind == KV_TASK_SWAP_IN_DELTA)) t.mask.assign(mask, mask + n);
  t.free_blocks = free_blocks;
  t.t_submit = Clock::now();
  {
    std::lock_guard<std::mutex> g(m->mu);
    if (m->stop) return KV_EBUSY;
    t.ticket = m->next_ticket++;
    if (ticket) *ticket = t.ticket;
    m->queue.push_back(std::move(t));
    m->st.submitted++;
  }
  m->cv_work.notify_one();
  return KV_OK;
}

int32_t kv_manager_poll(kv_manager_t* m, uint64_t* tickets, int32_t* status, int32_t cap, int32_t* n_out) {
  if (!m || !n_out || cap < 0 || (cap > 0 && !tickets)) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  harvest(m);
  int32_t k = 0;
  while (k < cap && !m->finished_order.empty()) {
    uint64_t tk = m->finished_order.front();
    m->finished_order.pop_front();
    auto f = m->finished.find(tk);
    if (f == m->finished.end()) continue;  // already taken by kv_manager_wait
    tickets[k] = tk;
    if (status) status[k] = f->second;
    m->finished.erase(f);
    ++k;
  }
  *n_out = k;
  return KV_OK;
}

int32_t kv_manager_wait(kv_manager_t* m, uint64_t ticket, int32_t* status) {
  if (!m || ticket == 0) return KV_EINVAL;
  std::unique_lock<std::mutex> lk(m->mu);
  if (ticket >= m->next_ticket) return KV_ENOENT;
  m->cv_done.wait(lk, [&] { return m->dispatched_upto >= ticket; });
  auto f = m->finished.find(ticket);
  if (f != m->finished.end()) {
    if (status) *status = f->second;
    m->finished.erase(f);
    return KV_OK;
  }
  for (size_t i = 0; i < m->flights.size(); ++i) {
    if (m->flights[i].ticket != ticket) continue;
    Flight f2 = m->flights[i];
    lk.unlock();
    // Synchronize (Algorithm 1, step 3.1 / step 4 "else" branch): block until the request's
    // last dispatched op is done
    int32_t rc = f2.status == KV_OK ? kv_wait(m->pool, f2.req) : KV_OK;
    lk.lock();
    for (size_t j = 0; j < m->flights.size(); ++j)
      if (m->flights[j].ticket == ticket) {
        m->flights.erase(m->flights.begin() + (long)j);
        break;
      }
    m->finished.erase(ticket);
    if (status) *status = f2.status;
    return rc;
  }
  return KV_ENOENT;  // reported earlier through poll or wait
}

int32_t kv_manager_drain(kv_manager_t* m) {
  if (!m) return KV_EINVAL;
  {
    std::unique_lock<std::mutex> lk(m->mu);
    const uint64_t last = m->next_ticket - 1;
    m->cv_done.wait(lk, [&] { return m->dispatched_upto >= last; });
  }
  return kv_wait_all(m->pool);
}

int32_t kv_manager_strategy(kv_manager_t* m, int32_t n_swap_in, int64_t swap_in_blocks, int32_t* async_out) {
  if (!m || !async_out || n_swap_in < 0 || swap_in_blocks < 0) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  // Estimated time of the swap-ins the scheduler wants now, and of a typical recent swap-in.
  // Short swap-ins are cheaper to wait for than to track across iterations (Section 3.2:
  // many short requests favour synchronous swap-in); long ones proceed asynchronously.
  const double now_ms = (double)swap_in_blocks * (double)m->record_bytes / (m->cfg.link_gbps * 1e6);
  double recent_blocks = 0;
  int recent_n = 0;
  for (const Recent& r : m->window)
    if (r.kind == KV_TASK_SWAP_IN || r.kind == KV_TASK_SWAP_IN_DELTA) {
      recent_blocks += (double)r.blocks;
      ++recent_n;
    }
  const double per_req_ms = n_swap_in > 0 ? now_ms / n_swap_in : 0.0;
  const double recent_ms =
      recent_n ? recent_blocks / recent_n * (double)m->record_bytes / (m->cfg.link_gbps * 1e6) : per_req_ms;
  // blend the current demand with the recent window so one outlier does not flip the mode
  const double typical_ms = 0.5 * (per_req_ms + recent_ms);
  *async_out = (n_swap_in > 0 && typical_ms >= m->cfg.sync_below_ms) ? 1 : 0;
  m->st.strategy_calls++;
  if (*async_out) m->st.strategy_async++;
  return KV_OK;
}

// ------------------------------------------------------------------------------------------
// Algorithm 1 as one call per scheduler iteration.
//
// The paper's listing executes swap-ins (step 2) before swap-outs (step 3) and then checks the
// two sets for a KV cache conflict (step 3.1).  On this library a conflict is a physical block
// that a swap-out of the iteration still has to read and a swap-in of the same iteration
// overwrites; the pool orders such a pair correctly on the device only if the reader was
// enqueued first.  The check is therefore made on the block tables before anything is
// dispatched: conflicting swap-outs go first (their gathers take well under a millisecond and
// the pool makes exactly the scatters concerned wait for them - the fine-grained
// Synchronize), everything else keeps the listing's order, swap-ins before swap-outs, which
// also keeps the host-to-device copies the scheduler waits for ahead of the iteration's
// device-to-host copies.
int32_t kv_manager_iterate(kv_manager_t* m, const kv_iteration_t* it, int64_t* resumed, int32_t cap,
                           int32_t* n_resumed, kv_iteration_result_t* res) {
  if (!m || !it || !n_resumed || cap < 0 || (cap > 0 && !resumed)) return KV_EINVAL;
  if (it->n_swap_in < 0 || it->n_swap_out < 0) return KV_EINVAL;
  if (it->n_swap_in > 0 && (!it->in_reqs || !it->in_n_blocks)) return KV_EINVAL;
  if (it->n_swap_out > 0 && (!it->out_reqs || !it->out_n_blocks)) return KV_EINVAL;
  kv_iteration_result_t r{};
  int32_t nres = 0;
  auto report = [&](int64_t req) {
    if (nres < cap) resumed[nres] = req;
    ++nres;
  };
  std::vector<int64_t> in_off((size_t)it->n_swap_in + 1, 0), out_off((size_t)it->n_swap_out + 1, 0);
  for (int32_t i = 0; i < it->n_swap_in; ++i) {
    if (it->in_n_blocks[i] < 0) return KV_EINVAL;
    in_off[(size_t)i + 1] = in_off[(size_t)i] + it->in_n_blocks[i];
  }
  for (int32_t i = 0; i < it->n_swap_out; ++i) {
    if (it->out_n_blocks[i] < 0) return KV_EINVAL;
    out_off[(size_t)i + 1] = out_off[(size_t)i] + it->out_n_blocks[i];
  }
  if ((in_off.back() > 0 && !it->in_tables) || (out_off.back() > 0 && !it->out_tables)) return KV_EINVAL;

  // ---- step 1: swap-ins of earlier iterations that have completed join the running requests
  {
    std::lock_guard<std::mutex> g(m->mu);
    harvest(m);
    auto settle = [&](std::vector<kv_manager::Pending>& list, bool is_in) {
      size_t w = 0;
      for (size_t i = 0; i < list.size(); ++i) {
        auto f = m->finished.find(list[i].ticket);
        if (f == m->finished.end()) {
          list[w++] = list[i];
          continue;
        }
        const int32_t status = f->second;
        m->finished.erase(f);
        if (status != KV_OK) {
          m->failures.push_back({list[i].req, status});
          m->where[list[i].req] = is_in ? kv_manager::SWAPPED : kv_manager::RUNNING;
        } else if (is_in) {
          m->where[list[i].req] = kv_manager::RUNNING;
          report(list[i].req);
          ++r.completed_swap_ins;
        }
      }
      list.resize(w);
    };
    settle(m->ongoing_swap_in, true);
    settle(m->pending_out, false);  // swap-outs only have failures to book
    while (!m->finished_order.empty() && !m->finished.count(m->finished_order.front())) m->finished_order.pop_front();
    // queue transitions of this iteration are checked before anything is dispatched
    for (int32_t i = 0; i < it->n_swap_in; ++i) {
      auto f = m->where.find(it->in_reqs[i]);
      if (f == m->where.end() || f->second != kv_manager::SWAPPED) return KV_ENOENT;  // not in `swapped`
    }
    for (int32_t i = 0; i < it->n_swap_out; ++i) {
      auto f = m->where.find(it->out_reqs[i]);
      if (f != m->where.end() && f->second != kv_manager::RUNNING) return KV_EBUSY;  // not in `running`
    }
  }

  // ---- step 3.1 (made first, see above): blocks named by a swap-out and by a swap-in
  std::vector<uint8_t> out_first((size_t)it->n_swap_out, 0);
  if (it->n_swap_in > 0 && it->n_swap_out > 0) {
    std::vector<int32_t> in_blocks(it->in_tables, it->in_tables + in_off.back());
    std::sort(in_blocks.begin(), in_blocks.end());
    for (int32_t i = 0; i < it->n_swap_out; ++i)
      for (int64_t k = out_off[(size_t)i]; k < out_off[(size_t)i + 1]; ++k)
        if (std::binary_search(in_blocks.begin(), in_blocks.end(), it->out_tables[k])) {
          out_first[(size_t)i] = 1;
          ++r.conflicts;
          break;
        }
  }
  std::vector<uint64_t> in_tickets((size_t)it->n_swap_in, 0), out_tickets((size_t)it->n_swap_out, 0);
  auto submit_out = [&](int32_t i) -> int32_t {
    const uint8_t* mask = it->out_dirty ? it->out_dirty + out_off[(size_t)i] : nullptr;
    return submit_task(m, mask ? KV_TASK_SWAP_OUT_DELTA : KV_TASK_SWAP_OUT, it->out_reqs[i],
                       it->out_tables + out_off[(size_t)i], it->out_n_blocks[i], mask,
                       &out_tickets[(size_t)i], (it->flags & KV_IT_FREE_OUT_BLOCKS) != 0);
  };
  int32_t rc;
  for (int32_t i = 0; i < it->n_swap_out; ++i)
    if (out_first[(size_t)i] && (rc = submit_out(i))) return rc;
  // ---- step 2: swap-ins
  int64_t in_blocks_total = 0;
  for (int32_t i = 0; i < it->n_swap_in; ++i) {
    if ((rc = kv_manager_submit(m, KV_TASK_SWAP_IN, it->in_reqs[i], it->in_tables + in_off[(size_t)i],
                                it->in_n_blocks[i], nullptr, &in_tickets[(size_t)i])))
      return rc;
    in_blocks_total += it->in_n_blocks[i];
  }
  // ---- step 3: swap-outs
  for (int32_t i = 0; i < it->n_swap_out; ++i)
    if (!out_first[(size_t)i] && (rc = submit_out(i))) return rc;

  // ---- step 4: asynchronous or synchronous swap-in
  int32_t async = 1;
  if (it->n_swap_in > 0 && (rc = kv_manager_strategy(m, it->n_swap_in, in_blocks_total, &async))) return rc;
  if (it->force_mode == 1) async = 1;
  if (it->force_mode == 2) async = 0;
  r.async = async;
  {
    std::lock_guard<std::mutex> g(m->mu);
    for (int32_t i = 0; i < it->n_swap_out; ++i) {
      m->where[it->out_reqs[i]] = kv_manager::SWAPPED;
      m->pending_out.push_back({it->out_reqs[i], out_tickets[(size_t)i]});
    }
    for (int32_t i = 0; i < it->n_swap_in; ++i) {
      m->where[it->in_reqs[i]] = kv_manager::ONGOING_SWAP_IN;
      if (async) m->ongoing_swap_in.push_back({it->in_reqs[i], in_tickets[(size_t)i]});
    }
  }
  if (!async) {  // SwapInStreamSynchronize: the scheduler stalls until they are back
    for (int32_t i = 0; i < it->n_swap_in; ++i) {
      int32_t status = KV_OK;
      rc = kv_manager_wait(m, in_tickets[(size_t)i], &status);
      std::lock_guard<std::mutex> g(m->mu);
      if (rc == KV_OK && status == KV_OK) {
        m->where[it->in_reqs[i]] = kv_manager::RUNNING;
        report(it->in_reqs[i]);
        ++r.waited_swap_ins;
      } else {
        m->where[it->in_reqs[i]] = kv_manager::SWAPPED;
        m->failures.push_back({it->in_reqs[i], rc != KV_OK ? rc : status});
      }
    }
  }
  {
    std::lock_guard<std::mutex> g(m->mu);
    r.ongoing_swap_ins = (int32_t)m->ongoing_swap_in.size();
    r.failures = (int32_t)m->failures.size();
    m->it_st.iterations++;
    m->it_st.swap_ins += it->n_swap_in;
    m->it_st.swap_outs += it->n_swap_out;
    m->it_st.async_iterations += (it->n_swap_in > 0 && async) ? 1 : 0;
    m->it_st.sync_iterations += (it->n_swap_in > 0 && !async) ? 1 : 0;
    m->it_st.conflicts += r.conflicts;
    m->it_st.resumed += nres;
  }
  *n_resumed = nres;
  if (res) *res = r;
  return KV_OK;
}

int32_t kv_manager_failures(kv_manager_t* m, int64_t* reqs, int32_t* status, int32_t cap, int32_t* n_out) {
  if (!m || !n_out || cap < 0 || (cap > 0 && (!reqs || !status))) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  int32_t k = 0;
  while (k < cap && !m->failures.empty()) {
    reqs[k] = m->failures.front().first;
    status[k] = m->failures.front().second;
    m->failures.erase(m->failures.begin());
    ++k;
  }
  *n_out = k;
  return KV_OK;
}

int32_t kv_manager_where(kv_manager_t* m, int64_t req, int32_t* where) {
  if (!m || !where) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  auto f = m->where.find(req);
  if (f == m->where.end()) return KV_ENOENT;
  *where = f->second;
  return KV_OK;
}

int32_t kv_manager_iteration_stats(kv_manager_t* m, kv_iteration_stats_t* out) {
  if (!m || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  *out = m->it_st;
  return KV_OK;
}

int32_t kv_manager_stats(kv_manager_t* m, kv_manager_stats_t* out) {
  if (!m || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  m->st.queued = (int64_t)m->queue.size();
  m->st.in_flight = (int64_t)m->flights.size();
  *out = m->st;
  return KV_OK;
}

}  // extern "C"
