// Host-side part of the C ABI: validation, capacity, workspace layout, error text.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cmath>
#include <cstring>
#include "moesys_internal.h"

namespace moesys {

static thread_local char g_err[512] = "";

int32_t fail(int32_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

int32_t check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return MOE_OK;
  return fail(MOE_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static std::atomic<int32_t> g_tuning[MOE_TUNE_COUNT] = {{0}, {1}, {0}, {0}};

int32_t tuning(int32_t key) { return g_tuning[key].load(std::memory_order_relaxed); }

static int32_t check_cfg(const moe_config* c) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "cfg is NULL");
  if (c->T < 0) return fail(MOE_ERR_INVALID_ARG, "T=%d is negative", c->T);
  if (c->d_model <= 0 || c->d_model % 64) return fail(MOE_ERR_INVALID_ARG, "d_model=%d must be a positive multiple of 64", c->d_model);
  if (c->d_ff <= 0 || c->d_ff % 64) return fail(MOE_ERR_INVALID_ARG, "d_ff=%d must be a positive multiple of 64", c->d_ff);
  if (c->E < 1 || c->E > MOE_MAX_EXPERTS) return fail(MOE_ERR_INVALID_ARG, "E=%d outside 1..%d", c->E, MOE_MAX_EXPERTS);
  if (c->k < 1 || c->k > c->E || c->k > MOE_MAX_TOPK) return fail(MOE_ERR_INVALID_ARG, "k=%d outside 1..min(E=%d,%d)", c->k, c->E, MOE_MAX_TOPK);
  if ((int64_t)c->k * c->T > (int64_t)INT32_MAX / 2) return fail(MOE_ERR_INVALID_ARG, "k*T=%lld too large", (long long)c->k * c->T);
  if (!(c->capacity_factor == c->capacity_factor) || std::isinf(c->capacity_factor)) return fail(MOE_ERR_INVALID_ARG, "capacity_factor is not finite");
  if (c->renormalize != 0 && c->renormalize != 1) return fail(MOE_ERR_INVALID_ARG, "renormalize=%d must be 0 or 1", c->renormalize);
  if (c->act != MOE_ACT_GELU && c->act != MOE_ACT_SWIGLU) return fail(MOE_ERR_INVALID_ARG, "act=%d unknown", c->act);
  if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "dtype=%d unknown", c->dtype);
  return MOE_OK;
}

// ceil(k*T*CF/E) without rounding: CF = m * 2^ex with a 24-bit integer m.
static int32_t capacity_of(const moe_config* c) {
  if (c->capacity_factor <= 0.f) return MOE_DROPLESS;
  int ex = 0;
  double fr = std::frexp((double)c->capacity_factor, &ex);   // CF = fr * 2^ex, 0.5 <= fr < 1
  unsigned __int128 m = (unsigned __int128)(uint64_t)std::ldexp(fr, 24);  // exact: float32 has 24 bits
  ex -= 24;
  unsigned __int128 num = (unsigned __int128)((uint64_t)c->k * (uint64_t)c->T) * m;
  unsigned __int128 den = (unsigned __int128)(uint64_t)c->E;
  if (ex >= 0) {
    if (ex > 40) return MOE_DROPLESS - 1;                       // astronomically large factor
    num <<= ex;
  } else {
    if (-ex > 100) { den = 0; }                                  // factor below 2^-76: quotient < 1
    else den <<= (-ex);
  }
  unsigned __int128 q = den == 0 ? 0 : (num + den - 1) / den;
  if (q < 1) q = 1;
  if (q > (unsigned __int128)(MOE_DROPLESS - 1)) q = MOE_DROPLESS - 1;
  return (int32_t)q;
}

int64_t max_rows(const moe_config* cfg) {
  int64_t A = (int64_t)cfg->k * cfg->T;
  int64_t C = capacity_of(cfg);
  int64_t cap = (int64_t)cfg->E * C;
  return A < cap ? A : cap;
}

size_t ffn_counter_offset(const moe_config* cfg) {
  return align_up((size_t)max_rows(cfg) * cfg->d_ff * elem_size(cfg->dtype), 256);
}

static void layout_of(const moe_config* c, moe_ws_layout* L) {
  const size_t s = elem_size(c->dtype);
  const size_t A = (size_t)c->k * (size_t)c->T;
  const size_t R = (size_t)max_rows(c);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L->topk_idx = take(A * 4);
  L->topk_w = take(A * 4);
  L->expert_counts = take((size_t)c->E * 4);
  L->expert_offsets = take((size_t)(c->E + 1) * 4);
  L->assign_to_row = take(A * 4);
  L->row_to_assign = take(A * 4);
  // segments that the bf16 path never writes are empty (the first GEMM gathers from x; with k = 1 the
  // second GEMM writes `out`)
  L->xd = take(gemm1_can_gather(c) ? 0 : R * c->d_model * s);
  L->h = take(R * c->d_ff * s);
  L->yd = take(gemm2_can_combine(c) ? 0 : R * c->d_model * s);
  L->scratch = take(((size_t)dispatch_blocks(c) + 1) * c->E * 4 + 256);
  L->tile_counters = take(TILE_COUNTER_INTS * 4);
  L->total = off;
  L->r_max = (int64_t)R;
}

int32_t check_weights(const moe_config* cfg, const moe_weights* w) {
  if (!w) return fail(MOE_ERR_INVALID_ARG, "weights is NULL");
  if (w->layout != MOE_LAYOUT_INPUT_MAJOR && w->layout != MOE_LAYOUT_OUTPUT_MAJOR)
    return fail(MOE_ERR_INVALID_ARG, "weights.layout=%d unknown", w->layout);
  if (cfg->act == MOE_ACT_GELU) {
    if (!w->w1 || !w->w2) return fail(MOE_ERR_INVALID_ARG, "GELU experts need w1 and w2");
  } else {
    if (!w->w_gate_proj || !w->w_up || !w->w_down)
      return fail(MOE_ERR_INVALID_ARG, "SwiGLU experts need w_gate_proj, w_up and w_down");
  }
  if (cfg->dtype == MOE_BF16 && w->layout != MOE_LAYOUT_OUTPUT_MAJOR)
    return fail(MOE_ERR_UNSUPPORTED, "bf16 experts must be MOE_LAYOUT_OUTPUT_MAJOR (use moe_transpose_expert_weights once)");
  if (w->expert_elem_offset && cfg->dtype != MOE_BF16)
    return fail(MOE_ERR_UNSUPPORTED, "per-expert offsets (expert_elem_offset) are supported for bf16 experts only");
  return MOE_OK;
}

}  // namespace moesys

using namespace moesys;

extern "C" {

const char* moe_status_string(int32_t st) {
  switch (st) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED: return "unsupported configuration";
    case MOE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MOE_ERR_HIP: return "HIP runtime error";
    case MOE_ERR_STATE: return "ring used out of order";
    default: return "unknown status";
  }
}

const char* moe_last_error(void) { return g_err; }
int32_t moe_version(void) { return 210; }

int32_t moe_set_tuning(int32_t key, int32_t value) {
  switch (key) {
    case MOE_TUNE_GEMM_TILE_ROWS:
      if (value != 0 && value != 256 && value != 320)
        return fail(MOE_ERR_INVALID_ARG, "moe_set_tuning: tile rows must be 0, 256 or 320 (got %d)", value);
      break;
    case MOE_TUNE_FEW_TOKEN_KERNELS:
      if (value != 0 && value != 1) return fail(MOE_ERR_INVALID_ARG, "moe_set_tuning: switch must be 0 or 1 (got %d)", value);
      break;
    case MOE_TUNE_GATE_TOKENS:
      if (value != 0 && value != 32 && value != 64 && value != 128)
        return fail(MOE_ERR_INVALID_ARG, "moe_set_tuning: gate tokens must be 0, 32, 64 or 128 (got %d)", value);
      break;
    case MOE_TUNE_GEMM_MFMA:
      if (value != 0 && value != 16 && value != 32)
        return fail(MOE_ERR_INVALID_ARG, "moe_set_tuning: the MFMA shape must be 0, 16 or 32 (got %d)", value);
      break;
    default: return fail(MOE_ERR_INVALID_ARG, "moe_set_tuning: key %d unknown", key);
  }
  g_tuning[key].store(value, std::memory_order_relaxed);
  return MOE_OK;
}

int32_t moe_get_tuning(int32_t key, int32_t* value) {
  if (key < 0 || key >= MOE_TUNE_COUNT || !value) return fail(MOE_ERR_INVALID_ARG, "moe_get_tuning: key %d unknown or value NULL", key);
  *value = tuning(key);
  return MOE_OK;
}
int32_t moe_config_check(const moe_config* cfg) { return check_cfg(cfg); }

int32_t moe_capacity(const moe_config* cfg) {
  if (check_cfg(cfg) != MOE_OK) return -1;
  return capacity_of(cfg);
}

size_t moe_workspace_bytes(const moe_config* cfg, int32_t kind) {
  if (check_cfg(cfg) != MOE_OK) return 0;
  moe_ws_layout L;
  layout_of(cfg, &L);
  switch (kind) {
    case MOE_WS_LAYER: return L.total;
    case MOE_WS_DISPATCH: return align_up(((size_t)dispatch_blocks(cfg) + 1) * cfg->E * 4 + 256, 256);
    case MOE_WS_FFN: return ffn_counter_offset(cfg) + align_up(TILE_COUNTER_INTS * 4, 256);
    default: fail(MOE_ERR_INVALID_ARG, "workspace kind %d unknown", kind); return 0;
  }
}

int32_t moe_workspace_layout(const moe_config* cfg, moe_ws_layout* out) {
  int32_t st = check_cfg(cfg);
  if (st != MOE_OK) return st;
  if (!out) return fail(MOE_ERR_INVALID_ARG, "out is NULL");
  layout_of(cfg, out);
  return MOE_OK;
}

}  // extern "C"
