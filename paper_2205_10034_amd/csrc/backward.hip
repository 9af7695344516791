// Backward pass of the expert FFN (GELU experts, bf16): the chain rule on
//   u = xd W1_e^T + b1_e,  h = gelu(u),  yd = h W2_e^T + b2_e        (weights OUTPUT_MAJOR [E, out, in])
// for the rows of every expert.  The paper's system is a training system (Section 3.2) and leaves the kernels
// open.  Products run on the grouped GEMM kernels: input gradients are plain grouped products on the
// INPUT_MAJOR copies of the weights (the contraction index of the transposed product is contiguous there),
// weight gradients contract over an expert's rows (grouped_wgrad_bf16.hip).  The pre-activations are
// recomputed rather than stored by the forward pass.  What is still separate from the GEMMs: the
// activation's derivative (one elementwise pass) and the bias gradients (column sums per expert).
#include "moesys_internal.h"

namespace moesys {

int32_t launch_grouped_matmul_bf16(const moe_config*, const void*, const void*, const void*, const int32_t*, void*, int, int,
                                   int32_t*, hipStream_t);
int32_t launch_wgrad_bf16(const uint16_t*, const uint16_t*, const int32_t*, float*, int, int, int, int64_t, hipStream_t);

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t to_bf16(float f) {  // round to nearest even (finite inputs)
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// d/du [u Phi(u)] = Phi(u) + u phi(u)
__device__ __forceinline__ float gelu_grad(float u) {
  return 0.5f * (1.f + erff(u * 0.70710678118654752f)) + u * expf(-0.5f * u * u) * 0.3989422804014327f;
}

// d_u = d_h * gelu'(u), in place on d_h; n8 = number of 8-element vectors
__global__ __launch_bounds__(256) void gelu_backward_kernel(uint4* __restrict__ dh, const uint4* __restrict__ u,
                                                            const int32_t* __restrict__ offsets, int E, size_t row_vec) {
  const size_t n8 = (size_t)offsets[E] * row_vec;  // only the kept rows
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    const uint4 a = dh[i], b = u[i];
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      o[q] = to_bf16(bf16_lo(aw[q]) * gelu_grad(bf16_lo(bw[q]))) | (to_bf16(bf16_hi(aw[q]) * gelu_grad(bf16_hi(bw[q]))) << 16);
    dh[i] = uint4{o[0], o[1], o[2], o[3]};
  }
}

// out[e, n] = sum over the rows r of expert e of d[r, n] (fp32).  One workgroup per (512-column block, expert):
// a lane owns 8 columns, the four wavefronts take every fourth row and meet in LDS (fixed order: results do
// not depend on scheduling).
__global__ __launch_bounds__(256) void bias_grad_kernel(const uint4* __restrict__ d, const int32_t* __restrict__ offsets,
                                                        float* __restrict__ out, int N) {
  __shared__ float part[4][512];
  const int e = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 512 + lane * 8;
  const int row_vec = N / 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < N) {
    for (int r = offsets[e] + wave; r < offsets[e + 1]; r += 4) {
      const uint4 v = d[(size_t)r * row_vec + col / 8];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) { acc[2 * q] += bf16_lo(w[q]); acc[2 * q + 1] += bf16_hi(w[q]); }
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) part[wave][lane * 8 + q] = acc[q];
  __syncthreads();
  for (int c = threadIdx.x; c < 512; c += 256)
    if (blockIdx.x * 512 + c < N)
      out[(size_t)e * N + blockIdx.x * 512 + c] = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
}

__global__ void clear8_kernel(int32_t* p) {
  if (threadIdx.x < 8) p[threadIdx.x] = 0;
}

}  // namespace
}  // namespace moesys

using namespace moesys;

extern "C" size_t moe_expert_ffn_backward_workspace_bytes(const moe_config* cfg) {
  if (moe_config_check(cfg) != MOE_OK) return 0;
  const size_t rf = align_up((size_t)max_rows(cfg) * cfg->d_ff * 2, 256);
  return 2 * rf + 256;  // u, d_h (becomes d_u), tile counters
}

extern "C" int32_t moe_expert_ffn_backward(const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                           const void* w2_input_major, const void* xd, const void* h, const void* d_yd,
                                           const int32_t* expert_offsets, void* d_xd, float* d_w1, float* d_b1,
                                           float* d_w2, float* d_b2, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if ((st = check_weights(cfg, w)) != MOE_OK) return st;
  if (cfg->dtype != MOE_BF16 || cfg->act != MOE_ACT_GELU)
    return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_backward: bf16 GELU experts only");
  if (w->expert_elem_offset) return fail(MOE_ERR_UNSUPPORTED, "moe_expert_ffn_backward: contiguous expert arrays only");
  if (!w1_input_major || !w2_input_major || !expert_offsets || !d_w1 || !d_w2)
    return fail(MOE_ERR_INVALID_ARG, "moe_expert_ffn_backward: NULL argument");
  if ((w->b1 && !d_b1) || (w->b2 && !d_b2)) return fail(MOE_ERR_INVALID_ARG, "moe_expert_ffn_backward: a bias without a gradient buffer");
  const size_t need = moe_expert_ffn_backward_workspace_bytes(cfg);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(MOE_ERR_WORKSPACE, "moe_expert_ffn_backward: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, ws_bytes);
  const int64_t rmax = max_rows(cfg);
  if (rmax > 0 && (!xd || !h || !d_yd || !d_xd)) return fail(MOE_ERR_INVALID_ARG, "moe_expert_ffn_backward: xd, h, d_yd, d_xd must be non-NULL");
  hipStream_t s = (hipStream_t)stream;
  const int E = cfg->E, d = cfg->d_model, f = cfg->d_ff;
  const size_t rf = align_up((size_t)rmax * f * 2, 256);
  char* base = (char*)ws;
  void* u = base;
  void* dh = base + rf;
  int32_t* ctr = (int32_t*)(base + 2 * rf);
  int64_t per_expert = rmax;
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS && C < per_expert) per_expert = C;
  auto clear = [&]() -> int32_t {
    hipLaunchKernelGGL(clear8_kernel, dim3(1), dim3(64), 0, s, ctr);
    return check_hip(hipGetLastError(), "counter clear launch");
  };
  // weight gradients that need nothing recomputed: dW2_e = d_yd_e^T h_e, db2_e = column sums of d_yd_e
  if ((st = launch_wgrad_bf16((const uint16_t*)d_yd, (const uint16_t*)h, expert_offsets, d_w2, E, d, f, per_expert, s)) != MOE_OK) return st;
  if (w->b2) {
    hipLaunchKernelGGL(bias_grad_kernel, dim3((d + 511) / 512, E), dim3(256), 0, s, (const uint4*)d_yd, expert_offsets, d_b2, d);
    if ((st = check_hip(hipGetLastError(), "bias gradient launch")) != MOE_OK) return st;
  }
  // u = xd W1^T + b1 (recomputed), d_h = d_yd W2, d_u = d_h * gelu'(u)   (without any row: every product
  // returns at once, the gradients come out as zeros)
  if ((st = clear()) != MOE_OK) return st;
  if ((st = launch_grouped_matmul_bf16(cfg, xd, w->w1, w->b1, expert_offsets, u, f, d, ctr, s)) != MOE_OK) return st;
  if ((st = clear()) != MOE_OK) return st;
  if ((st = launch_grouped_matmul_bf16(cfg, d_yd, w2_input_major, nullptr, expert_offsets, dh, f, d, ctr, s)) != MOE_OK) return st;
  hipLaunchKernelGGL(gelu_backward_kernel, dim3(2048), dim3(256), 0, s, (uint4*)dh, (const uint4*)u, expert_offsets, E, (size_t)f / 8);
  if ((st = check_hip(hipGetLastError(), "activation backward launch")) != MOE_OK) return st;
  // dW1_e = d_u_e^T xd_e, db1_e = column sums of d_u_e, d_xd = d_u W1
  if ((st = launch_wgrad_bf16((const uint16_t*)dh, (const uint16_t*)xd, expert_offsets, d_w1, E, f, d, per_expert, s)) != MOE_OK) return st;
  if (w->b1) {
    hipLaunchKernelGGL(bias_grad_kernel, dim3((f + 511) / 512, E), dim3(256), 0, s, (const uint4*)dh, expert_offsets, d_b1, f);
    if ((st = check_hip(hipGetLastError(), "bias gradient launch")) != MOE_OK) return st;
  }
  if ((st = clear()) != MOE_OK) return st;
  return launch_grouped_matmul_bf16(cfg, dh, w1_input_major, nullptr, expert_offsets, d_xd, d, f, ctr, s);
}
