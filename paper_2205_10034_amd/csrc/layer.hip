// moe_layer_forward: gate -> dispatch -> expert FFN -> combine on one stream with one workspace,
// and the stage timer used by the bench to attribute time per kernel group.
#include <new>
#include "moesys_internal.h"

struct moe_timer {
  hipEvent_t ev[MOE_STAGE_COUNT + 1];
  bool recorded;
};

namespace moesys {
namespace {

struct Segments {
  int32_t *topk_idx, *counts, *offsets, *a2r, *r2a, *tile_ctr;
  float* topk_w;
  void *xd, *h, *yd, *scratch;
};

// Validates what both halves of the layer need and resolves the workspace segments.
int32_t open_workspace(const char* who, const moe_config* cfg, const moe_weights* w, const void* x, void* ws,
                       size_t ws_bytes, Segments* sg) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (!w) return fail(MOE_ERR_INVALID_ARG, "%s: weights is NULL", who);
  if (cfg->T > 0 && !x) return fail(MOE_ERR_INVALID_ARG, "%s: x must be non-NULL", who);
  moe_ws_layout L;
  moe_workspace_layout(cfg, &L);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < L.total)
    return fail(MOE_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned (got %zu)", who, L.total, ws_bytes);
  char* base = (char*)ws;
  sg->topk_idx = (int32_t*)(base + L.topk_idx);
  sg->topk_w = (float*)(base + L.topk_w);
  sg->counts = (int32_t*)(base + L.expert_counts);
  sg->offsets = (int32_t*)(base + L.expert_offsets);
  sg->a2r = (int32_t*)(base + L.assign_to_row);
  sg->r2a = (int32_t*)(base + L.row_to_assign);
  sg->xd = base + L.xd;
  sg->h = base + L.h;
  sg->yd = base + L.yd;
  sg->scratch = base + L.scratch;
  sg->tile_ctr = (int32_t*)(base + L.tile_counters);
  return MOE_OK;
}

int32_t mark(moe_timer* timer, int i, hipStream_t s) {
  if (!timer) return MOE_OK;
  return check_hip(hipEventRecord(timer->ev[i], s), "hipEventRecord");
}

// gate -> dispatch bookkeeping (and, on the fp32 path, the dispatched copy)
int32_t route_impl(const char* who, const moe_config* cfg, const moe_weights* w, const void* x, void* ws,
                   size_t ws_bytes, hipStream_t s, moe_timer* timer) {
  Segments sg;
  int32_t st = open_workspace(who, cfg, w, x, ws, ws_bytes, &sg);
  if (st != MOE_OK) return st;
  if (!w->w_router) return fail(MOE_ERR_INVALID_ARG, "%s: w_router is NULL", who);
  if ((st = mark(timer, 0, s)) != MOE_OK) return st;
  const bool gather = gemm1_can_gather(cfg);
  if (gather && gate_dispatch_one_token_applies(cfg, w->w_router)) {
    // a step of one token: the gate's kernel writes the dispatch tables as well
    if ((st = launch_gate_dispatch_one_token(cfg, x, w->w_router, w->b_router, sg.topk_idx, sg.topk_w, sg.counts, sg.offsets,
                                             sg.a2r, sg.r2a, sg.tile_ctr, s)) != MOE_OK)
      return st;
    if ((st = mark(timer, 1, s)) != MOE_OK) return st;
    return mark(timer, 2, s);
  }
  if ((st = launch_gate_of(cfg, w, x, sg.topk_idx, sg.topk_w, nullptr, s)) != MOE_OK) return st;
  if ((st = mark(timer, 1, s)) != MOE_OK) return st;
  // bf16: the first GEMM gathers its rows from x through row_to_assign, so no dispatched copy is made
  if ((st = launch_dispatch(cfg, x, sg.topk_idx, sg.counts, sg.offsets, sg.a2r, sg.r2a, gather ? nullptr : sg.xd,
                            sg.scratch, sg.tile_ctr, s)) != MOE_OK)
    return st;
  return mark(timer, 2, s);
}

// expert FFN -> combine, from the routing tables in the workspace
int32_t experts_impl(const char* who, const moe_config* cfg, const moe_weights* w, const void* x, const void* residual,
                     void* out, void* ws, size_t ws_bytes, hipStream_t s, moe_timer* timer) {
  Segments sg;
  int32_t st = open_workspace(who, cfg, w, x, ws, ws_bytes, &sg);
  if (st != MOE_OK) return st;
  if ((st = check_weights(cfg, w)) != MOE_OK) return st;
  if (cfg->T > 0 && !out) return fail(MOE_ERR_INVALID_ARG, "%s: out must be non-NULL", who);
  if (out == x && residual != x) return fail(MOE_ERR_INVALID_ARG, "%s: out aliases x", who);
  const bool gather = gemm1_can_gather(cfg);
  if ((st = launch_gemm1(cfg, w, gather ? x : sg.xd, sg.offsets, sg.h, gather ? sg.r2a : nullptr, sg.tile_ctr, s)) != MOE_OK)
    return st;
  if ((st = mark(timer, 3, s)) != MOE_OK) return st;
  if (gemm2_can_combine(cfg)) {
    // one expert per token: the second GEMM scales each row by its gate weight, adds the residual and writes
    // it to its token's place; what is left of the combine stage are the rows of dropped tokens
    if ((st = launch_gemm2_combine(cfg, w, sg.h, sg.offsets, sg.r2a, sg.topk_w, residual, out, sg.tile_ctr, s)) != MOE_OK)
      return st;
    if ((st = mark(timer, 4, s)) != MOE_OK) return st;
    const int64_t C = moe_capacity(cfg);  // an expert gets at most T rows: no drops unless C is smaller
    if (C != MOE_DROPLESS && C < cfg->T)
      if ((st = launch_fill_dropped(cfg, sg.a2r, residual, out, s)) != MOE_OK) return st;
  } else if (expert_gemv_combine_one_token_applies(cfg)) {
    // a step of one token with several experts: the second product and the combine in one kernel (same yd, same out)
    const bool sw = cfg->act == MOE_ACT_SWIGLU;
    if ((st = launch_expert_gemv_combine_one_token(cfg, sg.h, sw ? w->w_down : w->w2, sw ? nullptr : w->b2, sg.offsets, sg.a2r,
                                                   sg.topk_w, residual, sg.yd, out, w->expert_elem_offset, s)) != MOE_OK)
      return st;
    if ((st = mark(timer, 4, s)) != MOE_OK) return st;
  } else {
    if ((st = launch_gemm2(cfg, w, sg.h, sg.offsets, sg.yd, sg.tile_ctr, s)) != MOE_OK) return st;
    if ((st = mark(timer, 4, s)) != MOE_OK) return st;
    if ((st = launch_combine(cfg, sg.yd, sg.a2r, sg.topk_w, residual, out, s)) != MOE_OK) return st;
  }
  if ((st = mark(timer, 5, s)) != MOE_OK) return st;
  if (timer) timer->recorded = true;
  return MOE_OK;
}

int32_t layer_impl(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual, void* out,
                   void* ws, size_t ws_bytes, hipStream_t s, moe_timer* timer) {
  // everything is validated before anything is launched
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if ((st = check_weights(cfg, w)) != MOE_OK) return st;
  if (cfg->T > 0 && (!x || !out)) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward: x and out must be non-NULL");
  if (out == x && residual != x) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward: out aliases x");
  if ((st = route_impl("moe_layer_forward", cfg, w, x, ws, ws_bytes, s, timer)) != MOE_OK) return st;
  return experts_impl("moe_layer_forward", cfg, w, x, residual, out, ws, ws_bytes, s, timer);
}

}  // namespace
}  // namespace moesys

using namespace moesys;

extern "C" {

int32_t moe_layer_forward(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual,
                          void* out, void* ws, size_t ws_bytes, void* stream) {
  return layer_impl(cfg, w, x, residual, out, ws, ws_bytes, (hipStream_t)stream, nullptr);
}

int32_t moe_layer_route(const moe_config* cfg, const moe_weights* w, const void* x, void* ws, size_t ws_bytes,
                        void* stream) {
  return route_impl("moe_layer_route", cfg, w, x, ws, ws_bytes, (hipStream_t)stream, nullptr);
}

int32_t moe_layer_experts(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual,
                          void* out, void* ws, size_t ws_bytes, void* stream) {
  return experts_impl("moe_layer_experts", cfg, w, x, residual, out, ws, ws_bytes, (hipStream_t)stream, nullptr);
}

int32_t moe_layer_forward_timed(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual,
                                void* out, void* ws, size_t ws_bytes, void* stream, moe_timer* timer) {
  if (!timer) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward_timed: timer is NULL");
  return layer_impl(cfg, w, x, residual, out, ws, ws_bytes, (hipStream_t)stream, timer);
}

int32_t moe_timer_create(moe_timer** out) {
  if (!out) return fail(MOE_ERR_INVALID_ARG, "moe_timer_create: out is NULL");
  moe_timer* t = new (std::nothrow) moe_timer();
  if (!t) return fail(MOE_ERR_HIP, "moe_timer_create: out of host memory");
  t->recorded = false;
  for (int i = 0; i <= MOE_STAGE_COUNT; ++i) {
    hipError_t e = hipEventCreate(&t->ev[i]);
    if (e != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(t->ev[j]);
      delete t;
      return check_hip(e, "hipEventCreate");
    }
  }
  *out = t;
  return MOE_OK;
}

int32_t moe_timer_destroy(moe_timer* t) {
  if (!t) return MOE_OK;
  for (int i = 0; i <= MOE_STAGE_COUNT; ++i) (void)hipEventDestroy(t->ev[i]);
  delete t;
  return MOE_OK;
}

int32_t moe_timer_read(moe_timer* t, float* stage_ms) {
  if (!t || !stage_ms) return fail(MOE_ERR_INVALID_ARG, "moe_timer_read: NULL argument");
  if (!t->recorded) return fail(MOE_ERR_STATE, "moe_timer_read: no timed call recorded");
  int32_t st = check_hip(hipEventSynchronize(t->ev[MOE_STAGE_COUNT]), "hipEventSynchronize");
  if (st != MOE_OK) return st;
  for (int i = 0; i < MOE_STAGE_COUNT; ++i) {
    st = check_hip(hipEventElapsedTime(&stage_ms[i], t->ev[i], t->ev[i + 1]), "hipEventElapsedTime");
    if (st != MOE_OK) return st;
  }
  return MOE_OK;
}

}  // extern "C"
