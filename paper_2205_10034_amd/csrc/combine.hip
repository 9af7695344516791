// Gate-weighted combine: out[t] = residual[t] + sum_j topk_w[t,j] * yd[assign_to_row[j*T+t]].
//
// The paper does not spell the combine out; it is the weighted un-permutation
// that the top-k gates it evaluates (Section 5.2) imply.  HBM-bound: one
// wavefront per token, 16-byte loads per lane, fp32 accumulation, one rounding.
#include "moesys_internal.h"

namespace moesys {
namespace {

__device__ __forceinline__ void unpack_bf16x8(const uint4& v, float (&o)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __uint_as_float(w[i] << 16);
    o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// float -> bfloat16 bits, round to nearest even (finite inputs; NaN kept quiet).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint4 pack_bf16x8(const float (&o)[8]) {
  uint4 v;
  v.x = f32_to_bf16_bits(o[0]) | (f32_to_bf16_bits(o[1]) << 16);
  v.y = f32_to_bf16_bits(o[2]) | (f32_to_bf16_bits(o[3]) << 16);
  v.z = f32_to_bf16_bits(o[4]) | (f32_to_bf16_bits(o[5]) << 16);
  v.w = f32_to_bf16_bits(o[6]) | (f32_to_bf16_bits(o[7]) << 16);
  return v;
}

template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ yd, const int32_t* __restrict__ a2r,
                                                      const float* __restrict__ topk_w, const uint4* residual,
                                                      uint4* out, int T, int k, int row_vec) {
  constexpr int PER = BF16 ? 8 : 4;
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int rows[MOE_MAX_TOPK];
  float w[MOE_MAX_TOPK];
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    rows[j] = j < k ? a2r[(size_t)j * T + t] : -1;
    w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
  }
  for (int v = lane; v < row_vec; v += 64) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    if (residual) {
      const uint4 r = residual[(size_t)t * row_vec + v];
      if (BF16) unpack_bf16x8(r, acc);
      else { acc[0] = __uint_as_float(r.x); acc[1] = __uint_as_float(r.y); acc[2] = __uint_as_float(r.z); acc[3] = __uint_as_float(r.w); }
    }
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
      if (rows[j] >= 0) {
        const uint4 y = yd[(size_t)rows[j] * row_vec + v];
        float yf[8];
        if (BF16) unpack_bf16x8(y, yf);
        else { yf[0] = __uint_as_float(y.x); yf[1] = __uint_as_float(y.y); yf[2] = __uint_as_float(y.z); yf[3] = __uint_as_float(y.w); }
#pragma unroll
        for (int i = 0; i < PER; ++i) acc[i] = fmaf(w[j], yf[i], acc[i]);
      }
    }
    uint4 o;
    if (BF16) o = pack_bf16x8(acc);
    else { o.x = __float_as_uint(acc[0]); o.y = __float_as_uint(acc[1]); o.z = __float_as_uint(acc[2]); o.w = __float_as_uint(acc[3]); }
    out[(size_t)t * row_vec + v] = o;
  }
}

// k = 1: rows of the tokens whose assignment was dropped (the others are written by the second GEMM).
__global__ __launch_bounds__(256) void fill_dropped_kernel(const int32_t* __restrict__ a2r, const uint4* residual, uint4* out,
                                                           int T, int row_vec) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T || a2r[t] >= 0) return;
  if (residual == out) return;  // in place: the row already holds its residual
  for (int v = lane; v < row_vec; v += 64)
    out[(size_t)t * row_vec + v] = residual ? residual[(size_t)t * row_vec + v] : uint4{0u, 0u, 0u, 0u};
}

// Backward of the combine: for every kept choice (t, j) with row r
//   d_yd[r] = topk_w[t,j] * d_out[t]          (rounded once to the activation dtype)
//   d_topk_w[t,j] = <d_out[t], yd[r]>         (fp32; 0 for a dropped choice)
// One wavefront per token: d_out[t] is read once, each of its rows of yd once; every row of d_yd is written
// by exactly one wavefront (a row belongs to one choice), so nothing is accumulated across wavefronts.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_backward_kernel(const uint4* __restrict__ d_out, const uint4* __restrict__ yd,
                                                               const int32_t* __restrict__ a2r,
                                                               const float* __restrict__ topk_w, uint4* __restrict__ d_yd,
                                                               float* __restrict__ d_topk_w, int T, int k, int row_vec) {
  constexpr int PER = BF16 ? 8 : 4;
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int rows[MOE_MAX_TOPK];
  float w[MOE_MAX_TOPK], dot[MOE_MAX_TOPK];
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    rows[j] = j < k ? a2r[(size_t)j * T + t] : -1;
    w[j] = j < k ? topk_w[(size_t)t * k + j] : 0.f;
    dot[j] = 0.f;
  }
  for (int v = lane; v < row_vec; v += 64) {
    const uint4 gv = d_out[(size_t)t * row_vec + v];
    float g[8];
    if (BF16) unpack_bf16x8(gv, g);
    else { g[0] = __uint_as_float(gv.x); g[1] = __uint_as_float(gv.y); g[2] = __uint_as_float(gv.z); g[3] = __uint_as_float(gv.w); }
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
      if (rows[j] >= 0) {
        const uint4 yv = yd[(size_t)rows[j] * row_vec + v];
        float y[8], o[8];
        if (BF16) unpack_bf16x8(yv, y);
        else { y[0] = __uint_as_float(yv.x); y[1] = __uint_as_float(yv.y); y[2] = __uint_as_float(yv.z); y[3] = __uint_as_float(yv.w); }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          dot[j] = fmaf(g[i], y[i], dot[j]);
          o[i] = w[j] * g[i];
        }
        uint4 ov;
        if (BF16) ov = pack_bf16x8(o);
        else { ov.x = __float_as_uint(o[0]); ov.y = __float_as_uint(o[1]); ov.z = __float_as_uint(o[2]); ov.w = __float_as_uint(o[3]); }
        d_yd[(size_t)rows[j] * row_vec + v] = ov;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    if (j < k) {
      float s = dot[j];
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
      if (lane == 0) d_topk_w[(size_t)t * k + j] = rows[j] >= 0 ? s : 0.f;
    }
  }
}

}  // namespace

int32_t launch_fill_dropped(const moe_config* cfg, const int32_t* a2r, const void* residual, void* out, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  const int row_vec = (int)((size_t)cfg->d_model * elem_size(cfg->dtype) / 16);
  hipLaunchKernelGGL(fill_dropped_kernel, dim3((cfg->T + 3) / 4), dim3(256), 0, s, a2r, (const uint4*)residual, (uint4*)out,
                     cfg->T, row_vec);
  return check_hip(hipGetLastError(), "fill launch");
}

int32_t launch_combine(const moe_config* cfg, const void* yd, const int32_t* a2r, const float* topk_w,
                       const void* residual, void* out, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  const int row_vec = (int)((size_t)cfg->d_model * elem_size(cfg->dtype) / 16);
  dim3 grid((cfg->T + 3) / 4), block(256);
  if (cfg->dtype == MOE_BF16)
    hipLaunchKernelGGL(combine_kernel<true>, grid, block, 0, s, (const uint4*)yd, a2r, topk_w,
                       (const uint4*)residual, (uint4*)out, cfg->T, cfg->k, row_vec);
  else
    hipLaunchKernelGGL(combine_kernel<false>, grid, block, 0, s, (const uint4*)yd, a2r, topk_w,
                       (const uint4*)residual, (uint4*)out, cfg->T, cfg->k, row_vec);
  return check_hip(hipGetLastError(), "combine launch");
}

}  // namespace moesys

using namespace moesys;

extern "C" int32_t moe_combine(const moe_config* cfg, const void* yd, const int32_t* assign_to_row,
                               const float* topk_w, const void* residual, void* out, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (cfg->T > 0 && (!assign_to_row || !topk_w || !out))
    return fail(MOE_ERR_INVALID_ARG, "moe_combine: assign_to_row, topk_w and out must be non-NULL");
  if (cfg->T > 0 && !yd && moesys::max_rows(cfg) > 0) return fail(MOE_ERR_INVALID_ARG, "moe_combine: yd is NULL");
  return launch_combine(cfg, yd, assign_to_row, topk_w, residual, out, (hipStream_t)stream);
}

extern "C" int32_t moe_combine_backward(const moe_config* cfg, const void* d_out, const void* yd,
                                        const int32_t* assign_to_row, const float* topk_w, void* d_yd,
                                        float* d_topk_w, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (cfg->T == 0) return MOE_OK;
  if (!d_out || !assign_to_row || !topk_w || !d_topk_w)
    return fail(MOE_ERR_INVALID_ARG, "moe_combine_backward: d_out, assign_to_row, topk_w and d_topk_w must be non-NULL");
  if (moesys::max_rows(cfg) > 0 && (!yd || !d_yd)) return fail(MOE_ERR_INVALID_ARG, "moe_combine_backward: yd and d_yd must be non-NULL");
  const int row_vec = (int)((size_t)cfg->d_model * elem_size(cfg->dtype) / 16);
  dim3 grid((cfg->T + 3) / 4), block(256);
  if (cfg->dtype == MOE_BF16)
    hipLaunchKernelGGL(combine_backward_kernel<true>, grid, block, 0, (hipStream_t)stream, (const uint4*)d_out, (const uint4*)yd,
                       assign_to_row, topk_w, (uint4*)d_yd, d_topk_w, cfg->T, cfg->k, row_vec);
  else
    hipLaunchKernelGGL(combine_backward_kernel<false>, grid, block, 0, (hipStream_t)stream, (const uint4*)d_out, (const uint4*)yd,
                       assign_to_row, topk_w, (uint4*)d_yd, d_topk_w, cfg->T, cfg->k, row_vec);
  return check_hip(hipGetLastError(), "combine backward launch");
}
