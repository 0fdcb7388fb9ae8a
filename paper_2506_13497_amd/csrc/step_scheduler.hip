// Host side of the paper's control plane that is driven by the step-time table this library is
// measured for (sections 4.2.3 and 5, greedy scheduling algorithm of the appendix): the optimal
// degree of parallelism B(r) from the change rate z, a buddy allocator of GPUs, and the greedy
// first-come-first-served scheduler that starts a request on what it can get, promotes "hungry"
// requests between denoising steps in the order of their starvation time, and scales a request
// down for the decoder.  No device code; integer microseconds throughout, so a run is exactly
// reproducible.  The rules, including what the paper leaves open, are stated with the
// declarations in ddit_hot.h.
#include "ddit_common.hpp"
#include "../../include/ddit_hot.h"

#include <algorithm>
#include <exception>
#include <new>
#include <set>
#include <utility>
#include <vector>

using ddit::set_error;

namespace {

constexpr int MAX_REQUESTS = 1 << 22;   // bounds the simulation's host memory (a few hundred bytes per request)

inline bool pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline int log2i(int64_t v) { int k = 0; while ((int64_t)1 << (k + 1) <= v) ++k; return k; }

// Buddy system over GPUs 0..n-1: one ordered set of free block starts per block size.
struct BuddyPool {
  int n, levels;
  std::vector<std::set<int>> free_;
  explicit BuddyPool(int n_gpus) : n(n_gpus), levels(log2i(n_gpus) + 1), free_(levels) { free_[levels - 1].insert(0); }
  // smallest free block that is large enough, lowest start; split keeping the lower half; -1 if none
  int alloc(int size) {
    const int k = log2i(size);
    int j = k;
    while (j < levels && free_[j].empty()) ++j;
    if (j >= levels) return -1;
    const int start = *free_[j].begin();
    free_[j].erase(free_[j].begin());
    while (j > k) { --j; free_[j].insert(start + (1 << j)); }
    return start;
  }
  void release(int start, int size) {
    int k = log2i(size);
    while (k < levels - 1) {
      auto it = free_[k].find(start ^ (1 << k));
      if (it == free_[k].end()) break;
      free_[k].erase(it);
      start &= ~(1 << k);
      ++k;
    }
    free_[k].insert(start);
  }
  bool is_allocated_block(int start, int size) const {
    // an aligned range is allocated as a whole iff no free block overlaps it (checked by the callers
    // that hand blocks back through the C ABI)
    for (int k = 0; k < levels; ++k)
      for (int s : free_[k])
        if (s < start + size && start < s + (1 << k)) return false;
    return true;
  }
  int free_gpus() const {
    int t = 0;
    for (int k = 0; k < levels; ++k) t += (int)free_[k].size() << k;
    return t;
  }
};

struct Running {
  std::vector<std::pair<int, int>> blocks;   // (start, size) in the order granted
  int p = 0, step = 0, last_step = 0;
  int64_t starv = 0, since = 0;
  bool in_vae = false, hungry = false;
};

int check_config(const ddit_sched_config *c) {
  if (!c) { set_error("config is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (c->struct_size != sizeof(ddit_sched_config)) {
    set_error("config->struct_size=%u, this library expects %zu", c->struct_size, sizeof(ddit_sched_config));
    return DDIT_ERR_INVALID_ARG;
  }
  if (!pow2(c->n_gpus) || c->n_gpus > 4096) { set_error("n_gpus=%d must be a power of two, at most 4096", c->n_gpus); return DDIT_ERR_INVALID_ARG; }
  if (c->n_steps < 1 || c->n_resolutions < 1 || c->n_dop < 1 || c->n_dop > 13) {
    set_error("n_steps=%d n_resolutions=%d n_dop=%d", c->n_steps, c->n_resolutions, c->n_dop);
    return DDIT_ERR_INVALID_ARG;
  }
  if (((int64_t)1 << (c->n_dop - 1)) > c->n_gpus) { set_error("the table's largest parallel size %d exceeds n_gpus=%d", 1 << (c->n_dop - 1), c->n_gpus); return DDIT_ERR_INVALID_ARG; }
  if (!c->step_us || !c->opt_dop) { set_error("step_us and opt_dop must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!pow2(c->vae_gpus)) { set_error("vae_gpus=%d must be a power of two", c->vae_gpus); return DDIT_ERR_INVALID_ARG; }
  for (int r = 0; r < c->n_resolutions; ++r) {
    if (!pow2(c->opt_dop[r]) || c->opt_dop[r] > (1 << (c->n_dop - 1))) {
      set_error("opt_dop[%d]=%d must be a power of two inside the table", r, c->opt_dop[r]);
      return DDIT_ERR_INVALID_ARG;
    }
    for (int k = 0; k < c->n_dop; ++k)
      if (c->step_us[(size_t)r * c->n_dop + k] < 1 || c->step_us[(size_t)r * c->n_dop + k] > ((int64_t)1 << 40)) {
        set_error("step_us[%d][%d]=%lld outside [1, 2^40]", r, k, (long long)c->step_us[(size_t)r * c->n_dop + k]);
        return DDIT_ERR_INVALID_ARG;
      }
    if (c->vae_us && (c->vae_us[r] < 0 || c->vae_us[r] > ((int64_t)1 << 40))) { set_error("vae_us[%d] outside [0, 2^40]", r); return DDIT_ERR_INVALID_ARG; }
  }
  return DDIT_OK;
}

}  // namespace

extern "C" {

int ddit_optimal_dop(const int64_t *step_us_row_host, int32_t n_dop, int64_t z_min_num, int64_t z_min_den,
                     int32_t *dop_out) {
  if (!step_us_row_host || !dop_out) { set_error("step_us_row and dop_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (n_dop < 1 || n_dop > 13 || z_min_den < 1 || z_min_num < 0 || z_min_num > ((int64_t)1 << 30) || z_min_den > ((int64_t)1 << 30)) {
    set_error("n_dop=%d z_min=%lld/%lld", n_dop, (long long)z_min_num, (long long)z_min_den);
    return DDIT_ERR_INVALID_ARG;
  }
  for (int k = 0; k < n_dop; ++k)
    if (step_us_row_host[k] < 1 || step_us_row_host[k] > ((int64_t)1 << 40)) { set_error("step time %d outside [1, 2^40]", k); return DDIT_ERR_INVALID_ARG; }
  // z(2^k) = 1 - t_k / t_{k-1}; all comparisons as exact cross products
  int best = 1;
  __int128 bn = 0, bd = 1;          // the best gain so far as (t_{k-1} - t_k) / t_{k-1}; starts at z_min
  bn = z_min_num; bd = z_min_den;
  for (int k = 1; k < n_dop; ++k) {
    const __int128 num = (__int128)step_us_row_host[k - 1] - step_us_row_host[k], den = step_us_row_host[k - 1];
    if (num * bd > bn * den) { best = 1 << k; bn = num; bd = den; }
  }
  *dop_out = best;
  return DDIT_OK;
}

static int ddit_buddy_create_impl(int32_t n_gpus, void **pool_out) {
  if (!pool_out) { set_error("pool_out is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!pow2(n_gpus) || n_gpus > 4096) { set_error("n_gpus=%d must be a power of two, at most 4096", n_gpus); return DDIT_ERR_INVALID_ARG; }
  BuddyPool *b = new BuddyPool(n_gpus);   // may throw: the caller below is guarded
  *pool_out = b;
  return DDIT_OK;
}

static int ddit_buddy_alloc_impl(void *pool, int32_t size, int32_t *start_out) {
  BuddyPool *b = reinterpret_cast<BuddyPool *>(pool);
  if (!b || !start_out) { set_error("pool and start_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!pow2(size) || size > b->n) { set_error("size=%d must be a power of two, at most %d", size, b->n); return DDIT_ERR_INVALID_ARG; }
  *start_out = b->alloc(size);
  return DDIT_OK;
}

static int ddit_buddy_release_impl(void *pool, int32_t start, int32_t size) {
  BuddyPool *b = reinterpret_cast<BuddyPool *>(pool);
  if (!b) { set_error("pool is NULL"); return DDIT_ERR_INVALID_ARG; }
  if (!pow2(size) || size > b->n || start < 0 || start % size || start + size > b->n) {
    set_error("block (%d, %d) is not an aligned block of the pool", start, size);
    return DDIT_ERR_INVALID_ARG;
  }
  if (!b->is_allocated_block(start, size)) { set_error("block (%d, %d) is not allocated as a whole", start, size); return DDIT_ERR_INVALID_ARG; }
  b->release(start, size);
  return DDIT_OK;
}

static int ddit_buddy_free_gpus_impl(void *pool, int32_t *free_out) {
  BuddyPool *b = reinterpret_cast<BuddyPool *>(pool);
  if (!b || !free_out) { set_error("pool and free_out must not be NULL"); return DDIT_ERR_INVALID_ARG; }
  *free_out = b->free_gpus();
  return DDIT_OK;
}

int ddit_buddy_destroy(void *pool) {
  delete reinterpret_cast<BuddyPool *>(pool);
  return DDIT_OK;
}

static int ddit_sched_simulate_impl(const ddit_sched_config *config, const ddit_sched_request *requests_host, int32_t n_requests,
                        ddit_sched_record *records_out, ddit_sched_event *events_out_or_null, int64_t max_events,
                        int64_t *n_events_out, ddit_sched_totals *totals_out) {
  int rc = check_config(config);
  if (rc != DDIT_OK) return rc;
  if (n_requests > MAX_REQUESTS) { set_error("n_requests=%d: at most %d requests per call", n_requests, MAX_REQUESTS); return DDIT_ERR_UNSUPPORTED; }
  if (n_requests < 0 || (n_requests > 0 && (!requests_host || !records_out))) { set_error("requests / records missing for n_requests=%d", n_requests); return DDIT_ERR_INVALID_ARG; }
  if (max_events < 0 || (max_events > 0 && !events_out_or_null)) { set_error("max_events=%lld without an event array", (long long)max_events); return DDIT_ERR_INVALID_ARG; }
  const ddit_sched_config &c = *config;
  for (int i = 0; i < n_requests; ++i) {
    const ddit_sched_request &q = requests_host[i];
    if (q.resolution < 0 || q.resolution >= c.n_resolutions) { set_error("requests[%d].resolution=%d outside the table", i, q.resolution); return DDIT_ERR_INVALID_ARG; }
    if (q.arrival_us < 0 || q.arrival_us > ((int64_t)1 << 50)) { set_error("requests[%d].arrival_us outside [0, 2^50]", i); return DDIT_ERR_INVALID_ARG; }
    if (i > 0 && q.arrival_us < requests_host[i - 1].arrival_us) { set_error("requests must be ordered by arrival time (index %d)", i); return DDIT_ERR_INVALID_ARG; }
  }
  auto t_step = [&](int r, int p) { return c.step_us[(size_t)r * c.n_dop + log2i(p)]; };
  auto vae = [&](int r) { return c.vae_us ? c.vae_us[r] : (int64_t)0; };

  BuddyPool pool(c.n_gpus);
  std::vector<Running> run(n_requests);
  std::set<std::pair<int64_t, int>> timeline;   // (time of the next step end / decoder end, request)
  std::vector<int> waiting, hungry;              // arrival order / order of becoming hungry
  int next_arrival = 0;
  bool released = false;
  int64_t now = 0, n_events = 0;
  __int128 occupancy = 0;

  auto emit = [&](int kind, int req, int start, int count) {
    if (n_events < max_events) {
      ddit_sched_event &e = events_out_or_null[n_events];
      e.time_us = now; e.kind = kind; e.request = req; e.gpu_start = start; e.gpu_count = count;
    }
    ++n_events;
  };
  auto hold = [&](int i) {
    occupancy += (__int128)run[i].p * (now - run[i].since);
    run[i].since = now;
  };
  auto give_back = [&](int i, int start, int size) { pool.release(start, size); emit(DDIT_SCHED_RELEASE, i, start, size); };
  auto drop_hungry = [&](int i) {
    run[i].hungry = false;
    hungry.erase(std::remove(hungry.begin(), hungry.end(), i), hungry.end());
  };
  for (int i = 0; i < n_requests; ++i) {
    ddit_sched_record &r = records_out[i];
    r.start_us = r.dit_end_us = r.end_us = -1; r.starvation = 0; r.first_dop = r.final_dop = r.promotions = 0;
  }

  while (next_arrival < n_requests || !timeline.empty()) {
    now = timeline.empty() ? requests_host[next_arrival].arrival_us : timeline.begin()->first;
    if (next_arrival < n_requests && requests_host[next_arrival].arrival_us < now) now = requests_host[next_arrival].arrival_us;
    // step ends and decoder ends of this microsecond, by request index (the set is ordered by (time, request))
    while (!timeline.empty() && timeline.begin()->first == now) {
      const int i = timeline.begin()->second;
      timeline.erase(timeline.begin());
      Running &s = run[i];
      const int r = requests_host[i].resolution;
      if (s.in_vae) {
        hold(i);
        give_back(i, s.blocks[0].first, s.blocks[0].second);
        records_out[i].end_us = now;
        s.blocks.clear(); s.p = 0;
        released = true;
        continue;
      }
      if (++s.step < c.n_steps) {
        timeline.insert({now + t_step(r, s.p), i});
        continue;
      }
      records_out[i].dit_end_us = now;
      records_out[i].final_dop = s.p;
      if (s.hungry) drop_hungry(i);
      int lowest = 0;
      for (size_t b = 1; b < s.blocks.size(); ++b)
        if (s.blocks[b].first < s.blocks[lowest].first) lowest = (int)b;
      emit(DDIT_SCHED_DIT_DONE, i, s.blocks[lowest].first, s.p);
      hold(i);
      if (vae(r) == 0) {
        for (const auto &b : s.blocks) give_back(i, b.first, b.second);
        records_out[i].end_us = now;
        s.blocks.clear(); s.p = 0;
      } else {
        const std::pair<int, int> low = s.blocks[lowest];
        for (size_t b = 0; b < s.blocks.size(); ++b)
          if ((int)b != lowest) give_back(i, s.blocks[b].first, s.blocks[b].second);
        int size = low.second;
        const int keep = std::min(c.vae_gpus, size);
        while (size > keep) { size /= 2; give_back(i, low.first + size, size); }
        s.blocks.assign(1, {low.first, size});
        s.p = size;
        s.in_vae = true;
        timeline.insert({now + vae(r), i});
      }
      released = true;
    }
    while (next_arrival < n_requests && requests_host[next_arrival].arrival_us == now) waiting.push_back(next_arrival++);
    // one scheduling pass: promotions (only after a release), then the waiting queue in arrival order
    if (released) {
      for (int i : hungry) {
        Running &s = run[i];
        const int r = requests_host[i].resolution;
        s.starv += (int64_t)(s.step - s.last_step) * (t_step(r, s.p) - t_step(r, c.opt_dop[r]));
        s.last_step = s.step;
        records_out[i].starvation = s.starv;
      }
      std::vector<int> order(hungry);
      std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        return run[a].starv != run[b].starv ? run[a].starv > run[b].starv : a < b;
      });
      for (int i : order) {
        Running &s = run[i];
        const int B = c.opt_dop[requests_host[i].resolution];
        bool grown = false;
        while (s.p < B) {
          const int start = pool.alloc(s.p);
          if (start < 0) break;
          if (!grown) { hold(i); grown = true; }
          s.blocks.push_back({start, s.p});
          emit(DDIT_SCHED_PROMOTE, i, start, s.p);
          s.p *= 2;
        }
        if (grown) {
          ++records_out[i].promotions;
          if (s.p == B) drop_hungry(i);
        }
      }
      released = false;
    }
    std::vector<int> still;
    for (int i : waiting) {
      const int r = requests_host[i].resolution;
      int p = c.opt_dop[r], start = -1;
      for (; p >= 1; p /= 2) {
        start = pool.alloc(p);
        if (start >= 0) break;
      }
      if (start < 0) { still.push_back(i); continue; }
      Running &s = run[i];
      s.blocks.assign(1, {start, p});
      s.p = p; s.since = now;
      records_out[i].start_us = now;
      records_out[i].first_dop = p;
      timeline.insert({now + t_step(r, p), i});
      emit(DDIT_SCHED_START, i, start, p);
      if (p < c.opt_dop[r]) { s.hungry = true; hungry.push_back(i); }
    }
    waiting.swap(still);
  }
  if (n_events_out) *n_events_out = n_events;
  if (totals_out) {
    if (occupancy > (__int128)INT64_MAX) { set_error("occupancy exceeds 63 bits"); return DDIT_ERR_UNSUPPORTED; }
    totals_out->occupancy_gpu_us = (int64_t)occupancy;
    totals_out->makespan_us = now;
  }
  return DDIT_OK;
}

// Nothing may throw across the C boundary: the containers above allocate host memory, so every call that
// touches them runs guarded and turns an exception into a status and an error text.
#define DDIT_GUARDED(call)                                                                       \
  try {                                                                                          \
    return call;                                                                                 \
  } catch (const std::bad_alloc &) {                                                             \
    set_error("out of host memory");                                                             \
    return DDIT_ERR_UNSUPPORTED;                                                                 \
  } catch (const std::exception &e) {                                                            \
    set_error("host exception: %s", e.what());                                                   \
    return DDIT_ERR_INVALID_ARG;                                                                 \
  } catch (...) {                                                                                \
    set_error("unknown host exception");                                                         \
    return DDIT_ERR_INVALID_ARG;                                                                 \
  }

int ddit_buddy_create(int32_t n_gpus, void **pool_out) { DDIT_GUARDED(ddit_buddy_create_impl(n_gpus, pool_out)) }
int ddit_buddy_alloc(void *pool, int32_t size, int32_t *start_out) { DDIT_GUARDED(ddit_buddy_alloc_impl(pool, size, start_out)) }
int ddit_buddy_release(void *pool, int32_t start, int32_t size) { DDIT_GUARDED(ddit_buddy_release_impl(pool, start, size)) }
int ddit_buddy_free_gpus(void *pool, int32_t *free_out) { DDIT_GUARDED(ddit_buddy_free_gpus_impl(pool, free_out)) }
int ddit_sched_simulate(const ddit_sched_config *config, const ddit_sched_request *requests_host, int32_t n_requests,
                        ddit_sched_record *records_out, ddit_sched_event *events_out_or_null, int64_t max_events,
                        int64_t *n_events_out, ddit_sched_totals *totals_out) {
  DDIT_GUARDED(ddit_sched_simulate_impl(config, requests_host, n_requests, records_out, events_out_or_null, max_events,
                                        n_events_out, totals_out))
}

}  // extern "C"
