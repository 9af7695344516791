// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "moesys.h"

namespace moesys {

// Records msg as this thread's last error and returns st.
int32_t fail(int32_t st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
int32_t check_hip(hipError_t e, const char* what);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t elem_size(int32_t dtype) { return dtype == MOE_BF16 ? 2 : 4; }

// Current value of a moe_tuning_key (moe_set_tuning).
int32_t tuning(int32_t key);

// Upper bound of dispatched rows: min(k*T, E*C).
int64_t max_rows(const moe_config* cfg);

// Number of blocks of DISPATCH_BLOCK assignments the bookkeeping kernels use.
constexpr int DISPATCH_BLOCK = 256;
inline int64_t dispatch_blocks(const moe_config* cfg) {
  int64_t A = (int64_t)cfg->k * cfg->T;
  return (A + DISPATCH_BLOCK - 1) / DISPATCH_BLOCK;
}

// The grouped GEMMs hand out their tiles through one counter per XCD: the first GEMM owns ints [0,8) of a
// 16-int block, the second [8,16).  A counter must be zero when its kernel starts: the dispatch stage
// clears the first GEMM's, the first GEMM clears the second's.
constexpr int TILE_COUNTER_INTS = 16;
// Byte offset of the counters inside an MOE_WS_FFN workspace (after h[R_max, d_ff]).
size_t ffn_counter_offset(const moe_config* cfg);

// Stage launchers (arguments already validated).
bool expert_gemv_combine_one_token_applies(const moe_config* cfg);
int32_t launch_expert_gemv_combine_one_token(const moe_config* cfg, const void* h, const void* w2, const void* bias,
                                             const int32_t* offsets, const int32_t* a2r, const float* topk_w,
                                             const void* residual, void* yd, void* out, const int64_t* eoff, hipStream_t s);
bool gate_dispatch_one_token_applies(const moe_config* cfg, const float* w_router);
int32_t launch_gate_dispatch_one_token(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                                       int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, int32_t* a2r,
                                       int32_t* r2a, int32_t* clear8, hipStream_t s);
int32_t launch_gate(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                    int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s);
// the same on the pre-split router when w carries one (moe_weights.w_router_packed) and it applies
int32_t launch_gate_of(const moe_config* cfg, const moe_weights* w, const void* x, int32_t* topk_idx, float* topk_w, float* probs,
                       hipStream_t s);
// clear8 (nullable): eight ints set to zero on the way (the first GEMM's tile counters).
int32_t launch_dispatch(const moe_config* cfg, const void* x, const int32_t* topk_idx, int32_t* counts,
                        int32_t* offsets, int32_t* a2r, int32_t* r2a, void* xd, void* ws, int32_t* clear8,
                        hipStream_t s);
// row_map (nullable, bf16 only): row_to_assign; xd is then x itself and the rows are gathered on the fly.
// tile_counters: the 16-int block above (bf16 only; the fp32 kernels ignore it).
int32_t launch_gemm1(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                     void* h, const int32_t* row_map, int32_t* tile_counters, hipStream_t s);
bool gemm1_can_gather(const moe_config* cfg);
int32_t launch_gemm2(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                     void* yd, int32_t* tile_counters, hipStream_t s);
// k = 1, bf16: the second GEMM writes out[t] = residual[t] + topk_w[t] * FFN row for every token that kept its
// expert; launch_fill_dropped writes the others (residual[t], or zero).  Together they replace
// launch_gemm2 + launch_combine and the dispatched-order output yd.
bool gemm2_can_combine(const moe_config* cfg);
int32_t launch_gemm2_combine(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                             const int32_t* r2a, const float* topk_w, const void* residual, void* out,
                             int32_t* tile_counters, hipStream_t s);
int32_t launch_fill_dropped(const moe_config* cfg, const int32_t* a2r, const void* residual, void* out, hipStream_t s);
int32_t launch_combine(const moe_config* cfg, const void* yd, const int32_t* a2r, const float* topk_w,
                       const void* residual, void* out, hipStream_t s);
int32_t check_weights(const moe_config* cfg, const moe_weights* w);

}  // namespace moesys
