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

// ---- the pool: policy + data movement ------------------------------------------------------------
//
// All experts' parameter blobs (one per layer and expert) stay in pinned host memory; a region of HBM is cut
// into slots of one blob each.  Before a layer's experts run, the caller hands over the per-expert row
// counts that the routing left on the device; every expert with rows is scheduled through the policy above
// (in ascending expert order, as one batch), the blobs of the misses are copied into their slots on the copy
// stream, the compute stream is made to wait for them, and the table of the experts' offsets inside the
// pool is written for the kernels (moe_weights.expert_elem_offset).  Traffic is proportional to the
// activated experts that are not yet resident, not to the layer: the case the ring of whole layers
// (Section 3.3.2) handles worst, few tokens per step.
//
// Reading the counts needs the host to wait for the compute stream, so by the time slots are reassigned
// every kernel that read them has finished; copies follow each other on the one copy stream.
struct moe_expert_pool {
  moe_expert_cache* policy;
  char* dev_pool;
  size_t slot_bytes, blob_bytes;
  int32_t n_layers, E;
  std::vector<const void*> host;   // [n_layers * E]
  hipStream_t copy_stream;
  bool own_stream;
  hipEvent_t copied;
  int32_t* counts_host;            // pinned [2][E]: the layer's counts, a prefetch's counts
  int64_t* offsets_host;           // pinned [E]
  uint64_t bytes_copied, copies, prefetched;
  bool copies_pending;             // copies enqueued since the compute stream last waited for the copy stream
};

extern "C" {

int32_t moe_expert_pool_create(void* dev_pool, size_t pool_bytes, size_t slot_bytes, const void* const* host_blobs,
                               int32_t n_layers, int32_t E, size_t blob_bytes, float threshold, float beta,
                               int32_t decay_steps, void* copy_stream, moe_expert_pool** out) {
  if (!out || !dev_pool || !host_blobs) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_create: NULL argument");
  if (n_layers < 1 || E < 1 || E > MOE_MAX_EXPERTS || blob_bytes == 0 || slot_bytes < blob_bytes || (slot_bytes & 255) ||
      ((uintptr_t)dev_pool & 255))
    return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_create: need n_layers, E >= 1, blob_bytes <= slot_bytes, "
                                     "slot_bytes and dev_pool multiples of 256");
  const size_t slots = pool_bytes / slot_bytes;
  if (slots < 1 || slots > (size_t)INT32_MAX) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_create: pool holds %zu slots", slots);
  for (int64_t i = 0; i < (int64_t)n_layers * E; ++i)
    if (!host_blobs[i]) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_create: host_blobs[%lld] is NULL", (long long)i);
  moe_expert_pool* p = new (std::nothrow) moe_expert_pool();
  if (!p) return fail(MOE_ERR_HIP, "moe_expert_pool_create: out of host memory");
  p->policy = nullptr;
  p->copy_stream = nullptr;
  p->own_stream = false;
  p->copied = nullptr;
  p->counts_host = nullptr;
  p->offsets_host = nullptr;
  int32_t st = moe_expert_cache_create(&p->policy, (int32_t)slots, threshold, beta, decay_steps);
  if (st == MOE_OK) {
    p->dev_pool = (char*)dev_pool;
    p->slot_bytes = slot_bytes;
    p->blob_bytes = blob_bytes;
    p->n_layers = n_layers;
    p->E = E;
    p->host.assign(host_blobs, host_blobs + (size_t)n_layers * E);
    p->bytes_copied = p->copies = p->prefetched = 0;
    p->copies_pending = false;
    if (copy_stream) {
      p->copy_stream = (hipStream_t)copy_stream;
    } else {
      st = check_hip(hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking), "hipStreamCreate");
      p->own_stream = st == MOE_OK;
    }
  }
  if (st == MOE_OK) st = check_hip(hipEventCreateWithFlags(&p->copied, hipEventDisableTiming), "hipEventCreate");
  if (st == MOE_OK) st = check_hip(hipHostMalloc((void**)&p->counts_host, sizeof(int32_t) * 2 * E, hipHostMallocDefault), "hipHostMalloc");
  if (st == MOE_OK) st = check_hip(hipHostMalloc((void**)&p->offsets_host, sizeof(int64_t) * E, hipHostMallocDefault), "hipHostMalloc");
  if (st != MOE_OK) {
    moe_expert_pool_destroy(p);
    return st;
  }
  *out = p;
  return MOE_OK;
}

int32_t moe_expert_pool_destroy(moe_expert_pool* p) {
  if (!p) return MOE_OK;
  if (p->copy_stream) (void)hipStreamSynchronize(p->copy_stream);
  if (p->copied) (void)hipEventDestroy(p->copied);
  if (p->own_stream && p->copy_stream) (void)hipStreamDestroy(p->copy_stream);
  if (p->counts_host) (void)hipHostFree(p->counts_host);
  if (p->offsets_host) (void)hipHostFree(p->offsets_host);
  moe_expert_cache_destroy(p->policy);
  delete p;
  return MOE_OK;
}

int32_t moe_expert_pool_prepare(moe_expert_pool* p, int32_t layer, const int32_t* counts_dev, int32_t elem_bytes,
                                int64_t* dev_offsets, void* compute_stream) {
  if (!p || !counts_dev || !dev_offsets) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_prepare: NULL argument");
  if (layer < 0 || layer >= p->n_layers) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_prepare: layer %d of %d", layer, p->n_layers);
  if ((elem_bytes != 2 && elem_bytes != 4) || p->slot_bytes % ((size_t)elem_bytes * 8))
    return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_prepare: elem_bytes must be 2 or 4 and divide the slot size into multiples of 8");
  hipStream_t cs = (hipStream_t)compute_stream;
  int32_t st = check_hip(hipMemcpyAsync(p->counts_host, counts_dev, sizeof(int32_t) * p->E, hipMemcpyDeviceToHost, cs), "hipMemcpyAsync(counts)");
  if (st != MOE_OK) return st;
  // the host needs the counts; everything enqueued before on the compute stream has finished after this
  if ((st = check_hip(hipStreamSynchronize(cs), "hipStreamSynchronize")) != MOE_OK) return st;
  if ((st = moe_expert_cache_begin_batch(p->policy)) != MOE_OK) return st;
  bool any_copy = false;
  for (int32_t e = 0; e < p->E; ++e) {
    p->offsets_host[e] = 0;
    if (p->counts_host[e] <= 0) continue;
    int32_t slot = -1, hit = 0;
    if ((st = moe_expert_cache_schedule(p->policy, (int64_t)layer * p->E + e, &slot, &hit, nullptr)) != MOE_OK) return st;
    p->offsets_host[e] = (int64_t)((size_t)slot * p->slot_bytes / (size_t)elem_bytes);
    if (!hit) {
      st = check_hip(hipMemcpyAsync(p->dev_pool + (size_t)slot * p->slot_bytes, p->host[(size_t)layer * p->E + e],
                                    p->blob_bytes, hipMemcpyHostToDevice, p->copy_stream), "hipMemcpyAsync(expert)");
      if (st != MOE_OK) return st;
      p->bytes_copied += p->blob_bytes;
      ++p->copies;
      any_copy = true;
    }
  }
  // (a prefetched blob may still be on its way: the event covers every copy enqueued so far)
  if (any_copy || p->copies_pending) {
    if ((st = check_hip(hipEventRecord(p->copied, p->copy_stream), "hipEventRecord")) != MOE_OK) return st;
    if ((st = check_hip(hipStreamWaitEvent(cs, p->copied, 0), "hipStreamWaitEvent")) != MOE_OK) return st;
    p->copies_pending = false;
  }
  return check_hip(hipMemcpyAsync(dev_offsets, p->offsets_host, sizeof(int64_t) * p->E, hipMemcpyHostToDevice, cs), "hipMemcpyAsync(offsets)");
}

int32_t moe_expert_pool_prefetch(moe_expert_pool* p, int32_t layer, const int32_t* counts_dev, void* stream,
                                 int32_t* n_copied) {
  if (!p || !counts_dev) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_prefetch: NULL argument");
  if (layer < 0 || layer >= p->n_layers) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_prefetch: layer %d of %d", layer, p->n_layers);
  hipStream_t ss = (hipStream_t)stream;
  int32_t* guess = p->counts_host + p->E;
  int32_t st = check_hip(hipMemcpyAsync(guess, counts_dev, sizeof(int32_t) * p->E, hipMemcpyDeviceToHost, ss), "hipMemcpyAsync(counts)");
  if (st != MOE_OK) return st;
  if ((st = check_hip(hipStreamSynchronize(ss), "hipStreamSynchronize")) != MOE_OK) return st;
  int32_t n = 0;
  for (int32_t e = 0; e < p->E; ++e) {
    if (guess[e] <= 0) continue;
    const int64_t item = (int64_t)layer * p->E + e;
    int32_t slot = -1;
    if ((st = moe_expert_cache_lookup(p->policy, item, &slot, nullptr)) != MOE_OK) return st;
    if (slot >= 0) continue;  // resident already: a guess is not a use, the counts stay as they are
    // a request inside the current batch: the experts of the layer that is running are not victims
    st = moe_expert_cache_schedule(p->policy, item, &slot, nullptr, nullptr);
    if (st == MOE_ERR_STATE) break;  // no slot outside the batch is left: stop guessing
    if (st != MOE_OK) return st;
    st = check_hip(hipMemcpyAsync(p->dev_pool + (size_t)slot * p->slot_bytes, p->host[(size_t)item], p->blob_bytes,
                                  hipMemcpyHostToDevice, p->copy_stream), "hipMemcpyAsync(expert)");
    if (st != MOE_OK) return st;
    p->bytes_copied += p->blob_bytes;
    ++p->copies;
    ++p->prefetched;
    p->copies_pending = true;
    ++n;
  }
  if (n_copied) *n_copied = n;
  return MOE_OK;
}

int32_t moe_expert_pool_stats(const moe_expert_pool* p, uint64_t* bytes_copied, uint64_t* copies, uint64_t* hits,
                              uint64_t* misses, uint64_t* evictions) {
  if (!p) return fail(MOE_ERR_INVALID_ARG, "moe_expert_pool_stats: pool is NULL");
  if (bytes_copied) *bytes_copied = p->bytes_copied;
  if (copies) *copies = p->copies;
  return moe_expert_cache_stats(p->policy, hits, misses, evictions);
}

}  // extern "C"

