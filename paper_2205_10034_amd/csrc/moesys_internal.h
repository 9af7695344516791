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

// Upper bound of dispatched rows: min(k*T, E*C).
int64_t max_rows(const moe_config* cfg);

// Number of blocks of DISPATCH_BLOCK assignments the bookkeeping kernels use.
constexpr int DISPATCH_BLOCK = 256;
inline int64_t dispatch_blocks(const moe_config* cfg) {
  int64_t A = (int64_t)cfg->k * cfg->T;
  return (A + DISPATCH_BLOCK - 1) / DISPATCH_BLOCK;
}

// Stage launchers (arguments already validated).
int32_t launch_gate(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                    int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s);
int32_t launch_dispatch(const moe_config* cfg, const void* x, const int32_t* topk_idx, int32_t* counts,
                        int32_t* offsets, int32_t* a2r, int32_t* r2a, void* xd, void* ws, hipStream_t s);
// row_map (nullable, bf16 only): row_to_assign; xd is then x itself and the rows are gathered on the fly.
int32_t launch_gemm1(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                     void* h, const int32_t* row_map, hipStream_t s);
bool gemm1_can_gather(const moe_config* cfg);
int32_t launch_gemm2(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                     void* yd, hipStream_t s);
int32_t launch_combine(const moe_config* cfg, const void* yd, const int32_t* a2r, const float* topk_w,
                       const void* residual, void* out, hipStream_t s);
int32_t check_weights(const moe_config* cfg, const moe_weights* w);

}  // namespace moesys
