// Ring memory offloading of expert parameters (Section 3.3.2).
//
// K sections of one HBM region hold the expert blobs of K of the N layers; the
// rest stay in pinned host memory.  After layer i has been computed its section
// is released and refilled, on a copy stream, with the blob of the layer K
// positions ahead, so that the copy overlaps the next layers' compute (the
// "calculation-released-load" procedure).  The g-th layer evaluation overall
// uses section g mod K, which keeps the mapping consistent when repeated
// inference steps wrap around and N is not a multiple of K.
//
// Ordering is carried by events only; no call here blocks the host except
// moe_ring_stats and moe_ring_destroy (which wait for the enqueued copies):
//   loaded[s]   recorded on the copy stream after section s has been filled;
//               moe_ring_acquire makes the compute stream wait for it
//   computed[s] recorded on the compute stream by moe_ring_release; the copy
//               stream waits for it before overwriting the section
#include <new>
#include <vector>
#include "moesys_internal.h"

using namespace moesys;

namespace {

int32_t hip_copy(void*, void* dst, const void* src, size_t bytes, void* stream) {
  return hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, (hipStream_t)stream) == hipSuccess ? 0 : 1;
}
int32_t hip_ev_create(void*, void** ev) {
  hipEvent_t e;
  if (hipEventCreate(&e) != hipSuccess) return 1;
  *ev = (void*)e;
  return 0;
}
int32_t hip_ev_destroy(void*, void* ev) { return hipEventDestroy((hipEvent_t)ev) == hipSuccess ? 0 : 1; }
int32_t hip_ev_record(void*, void* ev, void* stream) {
  return hipEventRecord((hipEvent_t)ev, (hipStream_t)stream) == hipSuccess ? 0 : 1;
}
int32_t hip_wait(void*, void* stream, void* ev) {
  return hipStreamWaitEvent((hipStream_t)stream, (hipEvent_t)ev, 0) == hipSuccess ? 0 : 1;
}
int32_t hip_ev_sync(void*, void* ev) { return hipEventSynchronize((hipEvent_t)ev) == hipSuccess ? 0 : 1; }
int32_t hip_ev_elapsed(void*, void* a, void* b, float* ms) {
  return hipEventElapsedTime(ms, (hipEvent_t)a, (hipEvent_t)b) == hipSuccess ? 0 : 1;
}

}  // namespace

struct moe_ring {
  moe_ring_backend be;
  bool hip_backend;
  char* dev_base;
  size_t layer_bytes;
  int32_t K, N;
  std::vector<const void*> host;
  void* copy_stream;
  bool own_stream;
  std::vector<void*> loaded, computed;               // per section
  std::vector<int32_t> resident;                     // layer held (or being loaded) per section
  std::vector<std::pair<void*, void*>> pending, idle; // start/stop event pairs around copies
  int64_t next_use;                                  // g: index of the next layer evaluation
  bool acquired;                                     // acquire(g) done, release pending
  uint64_t bytes_copied, copies;
  double copy_ms;
};

namespace {

// Reads the duration of every finished copy (waits for the unfinished ones) and recycles its events.
int32_t harvest(moe_ring* r) {
  for (auto& p : r->pending) {
    if (r->be.event_synchronize(r->be.user, p.second)) return fail(MOE_ERR_HIP, "ring: event synchronize failed");
    float ms = 0.f;
    if (r->be.event_elapsed_ms(r->be.user, p.first, p.second, &ms)) return fail(MOE_ERR_HIP, "ring: event elapsed failed");
    r->copy_ms += ms;
    r->idle.push_back(p);
  }
  r->pending.clear();
  return MOE_OK;
}

// Reads the duration of the oldest copy's event pair and recycles it (waits if that copy has not finished).
int32_t harvest_oldest(moe_ring* r) {
  const std::pair<void*, void*> p = r->pending.front();
  if (r->be.event_synchronize(r->be.user, p.second)) return fail(MOE_ERR_HIP, "ring: event synchronize failed");
  float ms = 0.f;
  if (r->be.event_elapsed_ms(r->be.user, p.first, p.second, &ms)) return fail(MOE_ERR_HIP, "ring: event elapsed failed");
  r->copy_ms += ms;
  r->idle.push_back(p);
  r->pending.erase(r->pending.begin());
  return MOE_OK;
}

int32_t enqueue_load(moe_ring* r, int layer, int s) {
  // A caller that never asks for the statistics must not grow the list without bound: beyond a few rings' worth
  // of copies the oldest pair is recycled here (its copy lies at least that many copies back on the one copy
  // stream, so it has normally long finished and the wait returns at once).
  if (r->pending.size() >= (size_t)4 * r->K + 16) {
    int32_t st = harvest_oldest(r);
    if (st != MOE_OK) return st;
  }
  std::pair<void*, void*> p{nullptr, nullptr};
  if (!r->idle.empty()) {
    p = r->idle.back();
    r->idle.pop_back();
  } else if (r->be.event_create(r->be.user, &p.first) || r->be.event_create(r->be.user, &p.second)) {
    if (p.first) r->be.event_destroy(r->be.user, p.first);
    return fail(MOE_ERR_HIP, "ring: event creation failed");
  }
  // the pair joins the pending list only once both of its events are recorded (a pair with an unrecorded stop
  // event could never be waited for)
  if (r->be.event_record(r->be.user, p.first, r->copy_stream)) {
    r->idle.push_back(p);
    return fail(MOE_ERR_HIP, "ring: event record failed");
  }
  if (r->be.copy_h2d_async(r->be.user, r->dev_base + (size_t)s * r->layer_bytes, r->host[layer], r->layer_bytes,
                           r->copy_stream)) {
    r->idle.push_back(p);
    return fail(MOE_ERR_HIP, "ring: host-to-device copy of layer %d failed", layer);
  }
  if (r->be.event_record(r->be.user, p.second, r->copy_stream)) {
    r->idle.push_back(p);
    return fail(MOE_ERR_HIP, "ring: event record failed");
  }
  r->pending.push_back(p);
  if (r->be.event_record(r->be.user, r->loaded[s], r->copy_stream)) return fail(MOE_ERR_HIP, "ring: event record failed");
  r->resident[s] = layer;
  r->bytes_copied += r->layer_bytes;
  r->copies += 1;
  return MOE_OK;
}

void free_events(moe_ring* r) {
  for (auto* v : {&r->loaded, &r->computed})
    for (void* e : *v)
      if (e) r->be.event_destroy(r->be.user, e);
  for (auto* v : {&r->pending, &r->idle})
    for (auto& p : *v) {
      r->be.event_destroy(r->be.user, p.first);
      r->be.event_destroy(r->be.user, p.second);
    }
}

}  // namespace

extern "C" {

int32_t moe_ring_create(void* dev_base, size_t budget_bytes, int32_t n_sections, const void* const* host_layers,
                        int32_t n_layers, size_t layer_bytes, void* copy_stream, const moe_ring_backend* backend,
                        moe_ring** out) {
  if (!out) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: out is NULL");
  *out = nullptr;
  if (!dev_base || ((uintptr_t)dev_base & 255)) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: dev_base NULL or not 256-byte aligned");
  if (n_sections < 1 || n_layers < 1 || layer_bytes == 0) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: n_sections, n_layers and layer_bytes must be positive");
  if (layer_bytes % 256) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: layer_bytes must be a multiple of 256");
  if (!host_layers) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: host_layers is NULL");
  for (int i = 0; i < n_layers; ++i)
    if (!host_layers[i]) return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: host_layers[%d] is NULL", i);
  const int32_t K = n_sections < n_layers ? n_sections : n_layers;
  if (budget_bytes / layer_bytes < (size_t)K)
    return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: budget of %zu bytes cannot hold %d sections of %zu bytes", budget_bytes, K, layer_bytes);
  if (backend && (!backend->copy_h2d_async || !backend->event_create || !backend->event_destroy || !backend->event_record ||
                  !backend->stream_wait_event || !backend->event_synchronize || !backend->event_elapsed_ms))
    return fail(MOE_ERR_INVALID_ARG, "moe_ring_create: backend has a NULL function");

  moe_ring* r = new (std::nothrow) moe_ring();
  if (!r) return fail(MOE_ERR_HIP, "moe_ring_create: out of host memory");
  r->hip_backend = backend == nullptr;
  if (backend) r->be = *backend;
  else r->be = moe_ring_backend{nullptr, hip_copy, hip_ev_create, hip_ev_destroy, hip_ev_record, hip_wait, hip_ev_sync, hip_ev_elapsed};
  r->dev_base = (char*)dev_base;
  r->layer_bytes = layer_bytes;
  r->K = K;
  r->N = n_layers;
  r->host.assign(host_layers, host_layers + n_layers);
  r->copy_stream = copy_stream;
  r->own_stream = false;
  r->next_use = 0;
  r->acquired = false;
  r->bytes_copied = r->copies = 0;
  r->copy_ms = 0.0;
  r->loaded.assign(K, nullptr);
  r->computed.assign(K, nullptr);
  r->resident.assign(K, -1);
  if (r->hip_backend && !copy_stream) {
    hipStream_t s;
    hipError_t e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);  // default priority
    if (e != hipSuccess) { delete r; return check_hip(e, "hipStreamCreateWithFlags"); }
    r->copy_stream = (void*)s;
    r->own_stream = true;
  }
  int32_t st = MOE_OK;
  for (int s = 0; s < K && st == MOE_OK; ++s)
    for (auto* v : {&r->loaded, &r->computed})
      if (r->be.event_create(r->be.user, &(*v)[s])) { st = fail(MOE_ERR_HIP, "moe_ring_create: event creation failed"); break; }
  for (int s = 0; s < K && st == MOE_OK; ++s) st = enqueue_load(r, s, s);  // preload layers 0..K-1
  if (st != MOE_OK) {
    free_events(r);
    if (r->own_stream) (void)hipStreamDestroy((hipStream_t)r->copy_stream);
    delete r;
    return st;
  }
  *out = r;
  return MOE_OK;
}

int32_t moe_ring_acquire(moe_ring* r, int32_t layer, void* compute_stream, const void** dev_ptr) {
  if (!r || !dev_ptr) return fail(MOE_ERR_INVALID_ARG, "moe_ring_acquire: NULL argument");
  const int32_t expect = (int32_t)(r->next_use % r->N);
  if (r->acquired) return fail(MOE_ERR_STATE, "moe_ring_acquire: layer %d was acquired and not yet released", expect);
  if (layer != expect) return fail(MOE_ERR_STATE, "moe_ring_acquire: layer %d requested, next in sequence is %d", layer, expect);
  const int s = (int)(r->next_use % r->K);
  if (r->resident[s] != layer) return fail(MOE_ERR_STATE, "moe_ring_acquire: section %d holds layer %d, not %d", s, r->resident[s], layer);
  if (r->be.stream_wait_event(r->be.user, compute_stream, r->loaded[s])) return fail(MOE_ERR_HIP, "moe_ring_acquire: stream wait failed");
  *dev_ptr = r->dev_base + (size_t)s * r->layer_bytes;
  r->acquired = true;
  return MOE_OK;
}

int32_t moe_ring_release(moe_ring* r, int32_t layer, void* compute_stream) {
  if (!r) return fail(MOE_ERR_INVALID_ARG, "moe_ring_release: ring is NULL");
  const int32_t expect = (int32_t)(r->next_use % r->N);
  if (!r->acquired || layer != expect) return fail(MOE_ERR_STATE, "moe_ring_release: layer %d is not the acquired layer", layer);
  const int s = (int)(r->next_use % r->K);
  r->acquired = false;
  r->next_use += 1;
  if (r->K >= r->N) return MOE_OK;  // everything resident: nothing to refill
  if (r->be.event_record(r->be.user, r->computed[s], compute_stream)) return fail(MOE_ERR_HIP, "moe_ring_release: event record failed");
  if (r->be.stream_wait_event(r->be.user, r->copy_stream, r->computed[s])) return fail(MOE_ERR_HIP, "moe_ring_release: stream wait failed");
  const int next_layer = (int)((r->next_use - 1 + r->K) % r->N);
  return enqueue_load(r, next_layer, s);
}

int32_t moe_ring_stats(moe_ring* r, uint64_t* bytes_copied, uint64_t* copies, double* copy_ms) {
  if (!r) return fail(MOE_ERR_INVALID_ARG, "moe_ring_stats: ring is NULL");
  int32_t st = harvest(r);
  if (st != MOE_OK) return st;
  if (bytes_copied) *bytes_copied = r->bytes_copied;
  if (copies) *copies = r->copies;
  if (copy_ms) *copy_ms = r->copy_ms;
  return MOE_OK;
}

int32_t moe_ring_destroy(moe_ring* r) {
  if (!r) return MOE_OK;
  for (auto& p : r->pending) r->be.event_synchronize(r->be.user, p.second);  // no copy may outlive the ring
  free_events(r);
  if (r->own_stream) (void)hipStreamDestroy((hipStream_t)r->copy_stream);
  delete r;
  return MOE_OK;
}

}  // extern "C"
