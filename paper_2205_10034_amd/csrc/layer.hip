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

int32_t layer_impl(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual, void* out,
                   void* ws, size_t ws_bytes, hipStream_t s, moe_timer* timer) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  st = check_weights(cfg, w);
  if (st != MOE_OK) return st;
  if (!w->w_router) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward: w_router is NULL");
  if (cfg->T > 0 && (!x || !out)) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward: x and out must be non-NULL");
  if (out == x && residual != x) return fail(MOE_ERR_INVALID_ARG, "moe_layer_forward: out aliases x");
  moe_ws_layout L;
  moe_workspace_layout(cfg, &L);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < L.total)
    return fail(MOE_ERR_WORKSPACE, "moe_layer_forward: workspace needs %zu bytes, 256-byte aligned (got %zu)", L.total, ws_bytes);
  char* base = (char*)ws;
  int32_t* topk_idx = (int32_t*)(base + L.topk_idx);
  float* topk_w = (float*)(base + L.topk_w);
  int32_t* counts = (int32_t*)(base + L.expert_counts);
  int32_t* offsets = (int32_t*)(base + L.expert_offsets);
  int32_t* a2r = (int32_t*)(base + L.assign_to_row);
  int32_t* r2a = (int32_t*)(base + L.row_to_assign);
  void* xd = base + L.xd;
  void* h = base + L.h;
  void* yd = base + L.yd;
  void* scratch = base + L.scratch;
  int32_t* tile_ctr = (int32_t*)(base + L.tile_counters);

  auto mark = [&](int i) -> int32_t {
    if (!timer) return MOE_OK;
    return check_hip(hipEventRecord(timer->ev[i], s), "hipEventRecord");
  };
  if ((st = mark(0)) != MOE_OK) return st;
  if ((st = launch_gate(cfg, x, w->w_router, w->b_router, topk_idx, topk_w, nullptr, s)) != MOE_OK) return st;
  if ((st = mark(1)) != MOE_OK) return st;
  // bf16: the first GEMM gathers its rows from x through row_to_assign, so no dispatched copy is made
  const bool gather = gemm1_can_gather(cfg);
  if ((st = launch_dispatch(cfg, x, topk_idx, counts, offsets, a2r, r2a, gather ? nullptr : xd, scratch, tile_ctr, s)) != MOE_OK) return st;
  if ((st = mark(2)) != MOE_OK) return st;
  if ((st = launch_gemm1(cfg, w, gather ? x : xd, offsets, h, gather ? r2a : nullptr, tile_ctr, s)) != MOE_OK) return st;
  if ((st = mark(3)) != MOE_OK) return st;
  if (gemm2_can_combine(cfg)) {
    // one expert per token: the second GEMM scales each row by its gate weight, adds the residual and writes
    // it to its token's place; what is left of the combine stage are the rows of dropped tokens
    if ((st = launch_gemm2_combine(cfg, w, h, offsets, r2a, topk_w, residual, out, tile_ctr, s)) != MOE_OK) return st;
    if ((st = mark(4)) != MOE_OK) return st;
    const int64_t C = moe_capacity(cfg);  // an expert gets at most T rows: no drops unless C is smaller
    if (C != MOE_DROPLESS && C < cfg->T)
      if ((st = launch_fill_dropped(cfg, a2r, residual, out, s)) != MOE_OK) return st;
  } else {
    if ((st = launch_gemm2(cfg, w, h, offsets, yd, tile_ctr, s)) != MOE_OK) return st;
    if ((st = mark(4)) != MOE_OK) return st;
    if ((st = launch_combine(cfg, yd, a2r, topk_w, residual, out, s)) != MOE_OK) return st;
  }
  if ((st = mark(5)) != MOE_OK) return st;
  if (timer) timer->recorded = true;
  return MOE_OK;
}

}  // namespace
}  // namespace moesys

using namespace moesys;

extern "C" {

int32_t moe_layer_forward(const moe_config* cfg, const moe_weights* w, const void* x, const void* residual,
                          void* out, void* ws, size_t ws_bytes, void* stream) {
  return layer_impl(cfg, w, x, residual, out, ws, ws_bytes, (hipStream_t)stream, nullptr);
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
