// Frequency-based cache of expert parameters: which experts stay in a pool of HBM slots.
//
// The policy is the paper's "Scheduling on Sparse Parameters" (Algorithm 2, Section 3.2.2), one memory
// tier up: the paper caches SSD-resident expert states in CPU memory; here pinned host memory is the
// slow tier and a pool of expert-sized HBM slots the cache.  Per request: a cached item's hit count
// grows by one; a new item takes a free slot while there is one; with the pool full, the item with the
// lowest hit count among those that reach the threshold gives up its slot.  Every `decay_steps`
// requests all counts are multiplied by `beta`.
//
// Where the printed algorithm is ambiguous: its free-space test `acc + 1 < size` is taken as
// `acc < size`; one item is evicted per request (ties: cached earliest); the victim is the lowest count
// among the items at or above the threshold (the prose), not "the overall minimum if it reaches the
// threshold" (the listing), which one decayed item would block for ever; and when no item reaches the
// threshold the lowest count overall goes, because an expert cannot be computed without a slot.
// Items requested since the last begin_batch are never victims: the experts of one layer evaluation
// are needed at the same time.
//
// Host code only; counts are doubles updated by the same operations in the same order as the test
// oracle's, so both take identical decisions.
#include <new>
#include <unordered_map>
#include <vector>
#include "moesys_internal.h"

using namespace moesys;

struct moe_expert_cache {
  struct Entry {
    int64_t item;
    double hits;
    int64_t cached_at;
    int64_t batch;
    bool used;
  };
  std::vector<Entry> slots;                       // slot -> entry
  std::unordered_map<int64_t, int32_t> where;     // item -> slot
  double threshold, beta;
  int32_t decay_steps, steps, filled;
  int64_t inserts, batch;
  uint64_t n_hits, n_misses, n_evictions;
};

extern "C" {

int32_t moe_expert_cache_create(moe_expert_cache** out, int32_t slots, float threshold, float beta,
                                int32_t decay_steps) {
  if (!out) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_create: out is NULL");
  if (slots < 1 || decay_steps < 1 || !(beta >= 0.f) || !(threshold == threshold))
    return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_create: slots >= 1, decay_steps >= 1, beta >= 0 required");
  moe_expert_cache* c = new (std::nothrow) moe_expert_cache();
  if (!c) return fail(MOE_ERR_HIP, "moe_expert_cache_create: out of host memory");
  c->slots.assign((size_t)slots, moe_expert_cache::Entry{-1, 0.0, 0, 0, false});
  c->threshold = (double)threshold;
  c->beta = (double)beta;
  c->decay_steps = decay_steps;
  c->steps = 0;
  c->filled = 0;
  c->inserts = 0;
  c->batch = 0;
  c->n_hits = c->n_misses = c->n_evictions = 0;
  *out = c;
  return MOE_OK;
}

int32_t moe_expert_cache_destroy(moe_expert_cache* c) {
  delete c;
  return MOE_OK;
}

int32_t moe_expert_cache_begin_batch(moe_expert_cache* c) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_begin_batch: cache is NULL");
  ++c->batch;
  return MOE_OK;
}

int32_t moe_expert_cache_schedule(moe_expert_cache* c, int64_t item, int32_t* slot, int32_t* hit, int64_t* evicted) {
  if (!c || !slot) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_schedule: cache and slot must be non-NULL");
  if (item < 0) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_schedule: item must be >= 0");
  int64_t gone = -1;
  int32_t s;
  auto it = c->where.find(item);
  const bool was_cached = it != c->where.end();
  if (was_cached) {
    s = it->second;
    c->slots[s].hits += 1.0;
    ++c->n_hits;
  } else {
    if (c->filled < (int32_t)c->slots.size()) {
      s = c->filled++;
    } else {
      // lowest count among the items at or above the threshold; if there is none, lowest count overall
      int32_t best = -1, best_any = -1;
      for (int32_t i = 0; i < (int32_t)c->slots.size(); ++i) {
        const auto& e = c->slots[i];
        if (e.batch == c->batch) continue;
        auto lower = [&](int32_t cur) {
          return cur < 0 || e.hits < c->slots[cur].hits ||
                 (e.hits == c->slots[cur].hits && e.cached_at < c->slots[cur].cached_at);
        };
        if (lower(best_any)) best_any = i;
        if (e.hits >= c->threshold && lower(best)) best = i;
      }
      s = best >= 0 ? best : best_any;
      if (s < 0)
        return fail(MOE_ERR_STATE, "moe_expert_cache_schedule: all %zu slots hold items of the current batch", c->slots.size());
      gone = c->slots[s].item;
      c->where.erase(gone);
      ++c->n_evictions;
    }
    c->slots[s] = moe_expert_cache::Entry{item, 1.0, c->inserts++, c->batch, true};
    c->where.emplace(item, s);
    ++c->n_misses;
  }
  c->slots[s].batch = c->batch;
  if (++c->steps == c->decay_steps) {
    for (int32_t i = 0; i < c->filled; ++i) c->slots[i].hits *= c->beta;
    c->steps = 0;
  }
  *slot = s;
  if (hit) *hit = was_cached ? 1 : 0;
  if (evicted) *evicted = gone;
  return MOE_OK;
}

int32_t moe_expert_cache_lookup(const moe_expert_cache* c, int64_t item, int32_t* slot, double* hits) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_lookup: cache is NULL");
  auto it = c->where.find(item);
  if (slot) *slot = it == c->where.end() ? -1 : it->second;
  if (hits) *hits = it == c->where.end() ? 0.0 : c->slots[it->second].hits;
  return MOE_OK;
}

int32_t moe_expert_cache_stats(const moe_expert_cache* c, uint64_t* hits, uint64_t* misses, uint64_t* evictions) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "moe_expert_cache_stats: cache is NULL");
  if (hits) *hits = c->n_hits;
  if (misses) *misses = c->n_misses;
  if (evictions) *evictions = c->n_evictions;
  return MOE_OK;
}

}  // extern "C"
