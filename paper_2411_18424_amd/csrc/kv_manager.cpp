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
};

namespace {

int32_t dispatch(kv_manager* m, Task& t) {
  const int32_t n = (int32_t)t.table.size();
  const int32_t* tab = n ? t.table.data() : nullptr;
  const uint8_t* mask = t.mask.empty() ? nullptr : t.mask.data();
  switch (t.kind) {
    case KV_TASK_SWAP_OUT:
      return swap_out(m->pool, t.req, tab, n);
    case KV_TASK_SWAP_IN:
      return swap_in(m->pool, t.req, tab, n);
    case KV_TASK_SWAP_OUT_DELTA:
      return swap_out_delta(m->pool, t.req, tab, n, mask, nullptr);
    case KV_TASK_SWAP_IN_DELTA:
      return swap_in_delta(m->pool, t.req, tab, n, mask, nullptr);
  }
  return KV_EINVAL;
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

int32_t kv_manager_submit(kv_manager_t* m, int32_t kind, int64_t req, const int32_t* table, int32_t n,
                          const uint8_t* mask, uint64_t* ticket) {
  if (!m || n < 0 || (n > 0 && !table) || kind < KV_TASK_SWAP_OUT || kind > KV_TASK_SWAP_IN_DELTA)
    return KV_EINVAL;
  if ((kind == KV_TASK_SWAP_OUT_DELTA || kind == KV_TASK_SWAP_IN_DELTA) && n > 0 && !mask) return KV_EINVAL;
  Task t;
  t.kind = kind;
  t.req = req;
  t.table.assign(table, table + n);
  if (mask && (kind == KV_TASK_SWAP_OUT_DELTA || kind == KV_TASK_SWAP_IN_DELTA)) t.mask.assign(mask, mask + n);
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

int32_t kv_manager_stats(kv_manager_t* m, kv_manager_stats_t* out) {
  if (!m || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(m->mu);
  m->st.queued = (int64_t)m->queue.size();
  m->st.in_flight = (int64_t)m->flights.size();
  *out = m->st;
  return KV_OK;
}

}  // extern "C"
