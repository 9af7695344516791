// Backward pass of the layer (bf16): the chain rule on the forward definition with the routing held fixed.
// Expert FFN, for the rows of every expert (weights OUTPUT_MAJOR [E, out, in]):
//   GELU    u = xd W1_e^T + b1_e,  h = gelu(u),  yd = h W2_e^T + b2_e
//   SwiGLU  g = xd Wg_e^T, u = xd Wu_e^T,  h = silu(g) * u,  yd = h Wd_e^T
// The paper's system is a training system (Section 3.2) and leaves the kernels open.  Products run on the
// grouped GEMM kernels: input gradients are plain grouped products on the INPUT_MAJOR copies of the weights
// (the contraction index of the transposed product is contiguous there), weight gradients contract over an
// expert's rows (grouped_wgrad_bf16.hip).  The pre-activations are recomputed rather than stored by the
// forward pass, by a product whose epilogue applies the activation's derivative to d_h; they never reach
// memory; the bias gradients (column sums per expert of d_yd and d_u) are by-products of the weight-gradient
// products that read those operands anyway.
#include "moesys_internal.h"

namespace moesys {

int32_t launch_gather_rows(const moe_config*, const void*, const int32_t*, void*, hipStream_t);
int32_t launch_grouped_matmul_bf16(const moe_config*, const void*, const void*, const void*, const int32_t*, void*, int, int,
                                   int32_t*, hipStream_t);
int32_t launch_gemm1_dgelu_bf16(const moe_config*, const void*, const void*, const void*, const int32_t*, const void*, void*,
                                int32_t*, hipStream_t);
int32_t launch_gemm1_dswiglu_bf16(const moe_config*, const void*, const void*, const void*, const int32_t*, const void*, void*,
                                  int32_t*, hipStream_t);
int32_t launch_wgrad_bf16(const uint16_t*, const uint16_t*, const int32_t*, void*, int, float*, int, int, int, int64_t, hipStream_t);

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t to_bf16(float f) {  // round to nearest even (finite inputs)
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Load-balancing auxiliary loss (the remedy for expert imbalance that the paper's Section 1 points to, in the
// form of the work cited there): L = coef * E * sum_e f_e * Pbar_e, f_e = fraction of the tokens whose first
// choice is expert e, Pbar_e = mean probability of e.  One workgroup per expert; fixed reduction order.
__global__ __launch_bounds__(256) void first_choice_fraction_kernel(const int32_t* __restrict__ topk_idx,
                                                                    const float* __restrict__ probs, float* __restrict__ f,
                                                                    float* __restrict__ pbar, int T, int E, int k) {
  __shared__ int cnt[256];
  __shared__ float sum[256];
  const int e = blockIdx.x;
  int c = 0;
  float a = 0.f;
  for (int t = threadIdx.x; t < T; t += 256) {
    c += topk_idx[(size_t)t * k] == e;
    if (probs) a += probs[(size_t)t * E + e];
  }
  cnt[threadIdx.x] = c;
  sum[threadIdx.x] = a;
  __syncthreads();
  for (int m = 128; m >= 1; m >>= 1) {
    if ((int)threadIdx.x < m) { cnt[threadIdx.x] += cnt[threadIdx.x + m]; sum[threadIdx.x] += sum[threadIdx.x + m]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    f[e] = (float)cnt[0] / (float)T;
    if (pbar) pbar[e] = sum[0] / (float)T;
  }
}

__global__ void aux_loss_kernel(const float* __restrict__ f, const float* __restrict__ pbar, float* __restrict__ loss, int E, float coef) {
  if (threadIdx.x || blockIdx.x) return;
  float a = 0.f;
  for (int e = 0; e < E; ++e) a = fmaf(f[e], pbar[e], a);
  *loss = coef * (float)E * a;
}

// d_z[t, e] = p[t,e] * (d_p[t,e] - sum_e' d_p[t,e'] p[t,e']).  d_p is, on the k selected experts,
// (d_w_j - sum_i d_w_i w_i) / S with S = sum of the selected probabilities if the weights are renormalised and
// d_w_j otherwise, zero elsewhere; plus, on every expert, aux_scale * f[e] (the auxiliary loss's gradient,
// aux_scale = coef * E / T; f NULL: none).  One wavefront per token, lanes over the experts.
__global__ __launch_bounds__(256) void gate_dlogits_kernel(const float* __restrict__ probs, const int32_t* __restrict__ topk_idx,
                                                           const float* __restrict__ topk_w, const float* __restrict__ d_topk_w,
                                                           float* __restrict__ d_z, int T, int E, int k, int renorm,
                                                           const float* __restrict__ f, float aux_scale) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  float S = 0.f, common = 0.f;
  for (int j = 0; j < k; ++j) {
    S += probs[(size_t)t * E + topk_idx[(size_t)t * k + j]];
    common += d_topk_w[(size_t)t * k + j] * topk_w[(size_t)t * k + j];
  }
  float s = 0.f;  // sum over the experts of d_p * p: the selected ones ...
  for (int j = 0; j < k; ++j) {
    const float dp = renorm ? (d_topk_w[(size_t)t * k + j] - common) / S : d_topk_w[(size_t)t * k + j];
    s += dp * probs[(size_t)t * E + topk_idx[(size_t)t * k + j]];
  }
  if (f) {  // ... and the auxiliary term on all of them (lanes in a fixed butterfly order)
    float a = 0.f;
    for (int e = lane; e < E; e += 64) a = fmaf(f[e], probs[(size_t)t * E + e], a);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) a += __shfl_xor(a, m, 64);
    s = fmaf(aux_scale, a, s);
  }
  for (int e = lane; e < E; e += 64) {
    float dp = 0.f;
    for (int j = 0; j < k; ++j)
      if (topk_idx[(size_t)t * k + j] == e) dp = renorm ? (d_topk_w[(size_t)t * k + j] - common) / S : d_topk_w[(size_t)t * k + j];
    if (f) dp = fmaf(aux_scale, f[e], dp);
    d_z[(size_t)t * E + e] = probs[(size_t)t * E + e] * (dp - s);
  }
}

// out[e] = sum_t d_z[t, e]: one workgroup per expert, fixed reduction order
__global__ __launch_bounds__(256) void gate_dbias_kernel(const float* __restrict__ d_z, float* __restrict__ out, int T, int E) {
  __shared__ float part[256];
  const int e = blockIdx.x;
  float acc = 0.f;
  for (int t = threadIdx.x; t < T; t += 256) acc += d_z[(size_t)t * E + e];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int m = 128; m >= 1; m >>= 1) {
    if ((int)threadIdx.x < m) part[threadIdx.x] += part[threadIdx.x + m];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[e] = part[0];
}

constexpr int DWG_SLICE = 64;  // (a multiple of 16) tokens per partial sum of the router's weight gradient (many slices: the kernel's
                               // parallelism is slices x column blocks)
constexpr int GB_TOK = 16;   // tokens per workgroup of dx_kernel (their loads are issued together)
constexpr int GB_MAXK = MOE_MAX_TOPK;  // choices per token

// d_x[t, i] = (extra[t, i]) + sum over the kept choices j of d_xd[a2r[j*T+t], i] + sum_e d_z[t,e] * W_g[i,e],
// rounded once.  A thread owns two columns i and keeps their router rows in registers across GB_TOK tokens.
template <int EC>
__global__ __launch_bounds__(256) void dx_kernel(const uint32_t* __restrict__ d_xd, const int32_t* __restrict__ a2r,
                                                 const float* __restrict__ d_z, const float* __restrict__ w_router,
                                                 const uint32_t* __restrict__ extra, uint32_t* __restrict__ d_x, int T, int d,
                                                 int E, int k) {
  // The tokens' d_z rows and dispatch rows go through LDS.  Read straight from memory they are the same for
  // every lane: E loads per token each, and row indices that the gathers would wait for one at a time.
  __shared__ float s_dz[GB_TOK][EC];
  __shared__ int32_t s_row[GB_MAXK][GB_TOK];
  const int t0 = blockIdx.y * GB_TOK;
  if ((int)threadIdx.x < k * GB_TOK) {
    const int j = threadIdx.x / GB_TOK, u = threadIdx.x % GB_TOK;
    s_row[j][u] = t0 + u < T ? a2r[(size_t)j * T + t0 + u] : -1;
  }
  __syncthreads();
  const bool active = (blockIdx.x * 256 + threadIdx.x) * 2 < (unsigned)d;
  const int i2 = active ? blockIdx.x * 256 + threadIdx.x : 0;  // column pair (idle threads redo pair 0, store nothing)
  // every load of the workgroup's tokens is issued before the first is used (the addresses are clamped into
  // the arrays; what a clamped load returns is discarded)
  uint32_t v[GB_TOK];
  const uint32_t* first = extra ? extra : d_xd;  // (without extra: row 0 of d_xd, a readable address; value unused)
#pragma unroll
  for (int u = 0; u < GB_TOK; ++u) v[u] = first[(extra ? (size_t)min(t0 + u, T - 1) * (d / 2) : (size_t)0) + i2];
  float a0[GB_TOK], a1[GB_TOK];
#pragma unroll
  for (int u = 0; u < GB_TOK; ++u) {
    a0[u] = extra ? bf16_lo(v[u]) : 0.f;
    a1[u] = extra ? bf16_hi(v[u]) : 0.f;
  }
  for (int j = 0; j < k; ++j) {
    int r[GB_TOK];
#pragma unroll
    for (int u = 0; u < GB_TOK; ++u) r[u] = s_row[j][u];
#pragma unroll
    for (int u = 0; u < GB_TOK; ++u) v[u] = d_xd[(size_t)max(r[u], 0) * (d / 2) + i2];
#pragma unroll
    for (int u = 0; u < GB_TOK; ++u) {
      a0[u] += r[u] >= 0 ? bf16_lo(v[u]) : 0.f;
      a1[u] += r[u] >= 0 ? bf16_hi(v[u]) : 0.f;
    }
  }
  // the gate's path, EC experts at a time: the thread keeps its two router rows' EC entries in registers
  for (int e0 = 0; e0 < E; e0 += EC) {
    if (e0) __syncthreads();  // (the previous chunk of s_dz has been read)
    for (int i = threadIdx.x; i < GB_TOK * EC; i += 256) {
      const int u = i / EC, e = e0 + i % EC;
      s_dz[u][i % EC] = (t0 + u < T && e < E) ? d_z[(size_t)(t0 + u) * E + e] : 0.f;
    }
    __syncthreads();
    float w0[EC], w1[EC];
    const float* wr = w_router + (size_t)(2 * i2) * E + e0;
    if (e0 + EC <= E && (E & 3) == 0 && (reinterpret_cast<uintptr_t>(w_router) & 15) == 0) {
      // 16-byte loads (a lane's rows share no cache line with another lane's, so the cost is per instruction)
#pragma unroll
      for (int q = 0; q < EC / 4; ++q) {
        const float4 p0 = reinterpret_cast<const float4*>(wr)[q], p1 = reinterpret_cast<const float4*>(wr + E)[q];
        w0[4 * q] = p0.x; w0[4 * q + 1] = p0.y; w0[4 * q + 2] = p0.z; w0[4 * q + 3] = p0.w;
        w1[4 * q] = p1.x; w1[4 * q + 1] = p1.y; w1[4 * q + 2] = p1.z; w1[4 * q + 3] = p1.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < EC; ++e) {
        w0[e] = e0 + e < E ? wr[e] : 0.f;
        w1[e] = e0 + e < E ? wr[E + e] : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < GB_TOK; ++u)
#pragma unroll
      for (int e = 0; e < EC; ++e) {
        a0[u] = fmaf(s_dz[u][e], w0[e], a0[u]);
        a1[u] = fmaf(s_dz[u][e], w1[e], a1[u]);
      }
  }
  if (active) {
#pragma unroll
    for (int u = 0; u < GB_TOK; ++u)
      if (t0 + u < T) d_x[(size_t)(t0 + u) * (d / 2) + i2] = to_bf16(a0[u]) | (to_bf16(a1[u]) << 16);
  }
}

// partial[slice, i, e] = sum over the slice's tokens of x[t, i] * d_z[t, e]; blockIdx.z: which EC experts
template <int EC>
__global__ __launch_bounds__(256) void dwg_partial_kernel(const uint32_t* __restrict__ x, const float* __restrict__ d_z,
                                                          float* __restrict__ partial, int T, int d, int E, int slice_tokens) {
  __shared__ float s_dz[DWG_SLICE][EC];
  const int ts = blockIdx.y * slice_tokens, e0 = blockIdx.z * EC;
  for (int i = threadIdx.x; i < slice_tokens * EC; i += 256) {
    const int u = i / EC, e = e0 + i % EC;
    s_dz[u][i % EC] = (ts + u < T && e < E) ? d_z[(size_t)(ts + u) * E + e] : 0.f;  // (zero rows past the last token)
  }
  __syncthreads();
  const int i2 = blockIdx.x * 256 + threadIdx.x;
  if (i2 * 2 >= d) return;
  float a0[EC], a1[EC];
#pragma unroll
  for (int e = 0; e < EC; ++e) a0[e] = a1[e] = 0.f;
  // the slice's tokens 16 at a time, their loads issued together (a workgroup per CU is all there is to hide
  // the latency of one load after another); tokens past the end re-read the last one against zero rows of s_dz
  for (int u0 = 0; u0 < slice_tokens; u0 += 16) {
    uint32_t v[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) v[q] = x[(size_t)min(ts + u0 + q, T - 1) * (d / 2) + i2];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const float x0 = bf16_lo(v[q]), x1 = bf16_hi(v[q]);
#pragma unroll
      for (int e = 0; e < EC; ++e) {
        a0[e] = fmaf(x0, s_dz[u0 + q][e], a0[e]);
        a1[e] = fmaf(x1, s_dz[u0 + q][e], a1[e]);
      }
    }
  }
  float* p0 = partial + ((size_t)blockIdx.y * d + 2 * i2) * E + e0;
#pragma unroll
  for (int e = 0; e < EC; ++e)
    if (e0 + e < E) { p0[e] = a0[e]; p0[E + e] = a1[e]; }
}

// out[n] = sum over the slices of partial[slice, n], in slice order
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ partial, float* __restrict__ out, size_t n, int slices) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
#pragma unroll 8
  for (int s = 0; s < slices; ++s) acc += partial[(size_t)s * n + i];
  out[i] = acc;
}

__global__ void clear_counters_kernel(int32_t* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0;
}

}  // namespace
}  // namespace moesys

using namespace moesys;

extern "C" size_t moe_expert_ffn_backward_workspace_bytes(const moe_config* cfg) {
  if (moe_config_check(cfg) != MOE_OK) return 0;
  const size_t rf = align_up((size_t)max_rows(cfg) * cfg->d_ff * 2, 256);
  // GELU: d_h (becomes d_u); SwiGLU: d_h and [d_g | d_u]; three blocks of tile counters
  return (cfg->act == MOE_ACT_SWIGLU ? 3 : 1) * rf + 256;
}

static int32_t ffn_backward_impl(const char* who, const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                 const void* w2_input_major, const void* xd, const void* h, const void* d_yd,
                                 const int32_t* expert_offsets, void* d_xd, void* d_w1, float* d_b1, void* d_w2,
                                 float* d_b2, int32_t d_w_dtype, void* ws, size_t ws_bytes, void* stream);

extern "C" int32_t moe_expert_ffn_backward(const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                           const void* w2_input_major, const void* xd, const void* h, const void* d_yd,
                                           const int32_t* expert_offsets, void* d_xd, void* d_w1, float* d_b1,
                                           void* d_w2, float* d_b2, int32_t d_w_dtype, void* ws, size_t ws_bytes,
                                           void* stream) {
  return ffn_backward_impl("moe_expert_ffn_backward", cfg, w, w1_input_major, w2_input_major, xd, h, d_yd, expert_offsets,
                           d_xd, d_w1, d_b1, d_w2, d_b2, d_w_dtype, ws, ws_bytes, stream);
}

static int32_t ffn_backward_impl(const char* who, const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                 const void* w2_input_major, const void* xd, const void* h, const void* d_yd,
                                 const int32_t* expert_offsets, void* d_xd, void* d_w1, float* d_b1, void* d_w2,
                                 float* d_b2, int32_t d_w_dtype, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (d_w_dtype != MOE_F32 && d_w_dtype != MOE_BF16)
    return fail(MOE_ERR_INVALID_ARG, "%s: the weight gradients are MOE_F32 or MOE_BF16 (got %d)", who, d_w_dtype);
  if (st != MOE_OK) return st;
  if ((st = check_weights(cfg, w)) != MOE_OK) return st;
  if (cfg->dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "%s: bf16 only", who);
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  if (w->expert_elem_offset) return fail(MOE_ERR_UNSUPPORTED, "%s: contiguous expert arrays only", who);
  if (!w1_input_major || !w2_input_major || !expert_offsets || !d_w1 || !d_w2)
    return fail(MOE_ERR_INVALID_ARG, "%s: NULL argument", who);
  if (!sw && ((w->b1 && !d_b1) || (w->b2 && !d_b2))) return fail(MOE_ERR_INVALID_ARG, "%s: a bias without a gradient buffer", who);
  const size_t need = moe_expert_ffn_backward_workspace_bytes(cfg);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(MOE_ERR_WORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned (got %zu)", who, need, ws_bytes);
  const int64_t rmax = max_rows(cfg);
  if (rmax > 0 && (!xd || !h || !d_yd || !d_xd)) return fail(MOE_ERR_INVALID_ARG, "%s: xd, h, d_yd, d_xd must be non-NULL", who);
  hipStream_t s = (hipStream_t)stream;
  const int E = cfg->E, d = cfg->d_model, f = cfg->d_ff;
  const size_t rf = align_up((size_t)rmax * f * 2, 256);
  char* base = (char*)ws;
  void* dh = base;
  int32_t* ctr = (int32_t*)(base + (sw ? 3 : 1) * rf);
  int64_t per_expert = rmax;
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS && C < per_expert) per_expert = C;
  // every product draws its tiles from eight zeroed counters of its own
  hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, s, ctr, 24);
  if ((st = check_hip(hipGetLastError(), "counter clear launch")) != MOE_OK) return st;
  // weight gradients that need nothing recomputed: dW2_e = d_yd_e^T h_e, with db2_e = column sums of d_yd_e on the side
  if ((st = launch_wgrad_bf16((const uint16_t*)d_yd, (const uint16_t*)h, expert_offsets, d_w2, d_w_dtype, (!sw && w->b2) ? d_b2 : nullptr, E, d, f,
                              per_expert, s)) != MOE_OK) return st;
  if (sw) {
    // d_h = d_yd W_down; [d_g | d_u] from d_h and the recomputed gate and up products; the gradient of the
    // stacked [W_gate; W_up] in one product, d_xd in one product over the 2 d_ff columns of [d_g | d_u]
    void* dgu = base + rf;
    if ((st = launch_grouped_matmul_bf16(cfg, d_yd, w2_input_major, nullptr, expert_offsets, dh, f, d, ctr, s)) != MOE_OK) return st;
    if ((st = launch_gemm1_dswiglu_bf16(cfg, xd, w->w_gate_proj, w->w_up, expert_offsets, dh, dgu, ctr + 8, s)) != MOE_OK) return st;
    if ((st = launch_wgrad_bf16((const uint16_t*)dgu, (const uint16_t*)xd, expert_offsets, d_w1, d_w_dtype, nullptr, E, 2 * f, d, per_expert, s)) != MOE_OK) return st;
    return launch_grouped_matmul_bf16(cfg, dgu, w1_input_major, nullptr, expert_offsets, d_xd, d, 2 * f, ctr + 16, s);
  }
  // d_h = d_yd W2, then d_u = d_h * gelu'(u) in place, u = xd W1^T + b1 being recomputed by the product whose
  // epilogue applies the derivative: the pre-activations never reach memory.  (Without any row every product
  // returns at once and the gradients come out as zeros.)
  if ((st = launch_grouped_matmul_bf16(cfg, d_yd, w2_input_major, nullptr, expert_offsets, dh, f, d, ctr, s)) != MOE_OK) return st;
  if ((st = launch_gemm1_dgelu_bf16(cfg, xd, w->w1, w->b1, expert_offsets, dh, dh, ctr + 8, s)) != MOE_OK) return st;
  // dW1_e = d_u_e^T xd_e (db1_e = column sums of d_u_e on the side), d_xd = d_u W1
  if ((st = launch_wgrad_bf16((const uint16_t*)dh, (const uint16_t*)xd, expert_offsets, d_w1, d_w_dtype, w->b1 ? d_b1 : nullptr, E, f, d, per_expert,
                              s)) != MOE_OK) return st;
  return launch_grouped_matmul_bf16(cfg, dh, w1_input_major, nullptr, expert_offsets, d_xd, d, f, ctr + 16, s);
}

extern "C" int32_t moe_gate_aux_loss(const moe_config* cfg, const float* probs, const int32_t* topk_idx, float coef,
                                     float* expert_fraction, float* mean_prob, float* loss, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (!expert_fraction || !mean_prob || !loss) return fail(MOE_ERR_INVALID_ARG, "moe_gate_aux_loss: NULL output");
  if (cfg->T == 0) return fail(MOE_ERR_INVALID_ARG, "moe_gate_aux_loss: no tokens (the loss is a mean over tokens)");
  if (!probs || !topk_idx) return fail(MOE_ERR_INVALID_ARG, "moe_gate_aux_loss: NULL input");
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(first_choice_fraction_kernel, dim3(cfg->E), dim3(256), 0, s, topk_idx, probs, expert_fraction, mean_prob, cfg->T,
                     cfg->E, cfg->k);
  hipLaunchKernelGGL(aux_loss_kernel, dim3(1), dim3(64), 0, s, (const float*)expert_fraction, (const float*)mean_prob, loss, cfg->E, coef);
  return check_hip(hipGetLastError(), "moe_gate_aux_loss");
}

// ---- whole layer ------------------------------------------------------------------------------------
namespace {

struct BwLayout {
  size_t probs, idx, w, d_w, d_z, frac, xd, d_yd, d_xd, yd, partial, ffn, total;
  int slices;
};


void bw_layout(const moe_config* cfg, BwLayout* L) {
  const size_t T = (size_t)cfg->T, E = (size_t)cfg->E, k = (size_t)cfg->k, d = (size_t)cfg->d_model;
  const size_t R = (size_t)max_rows(cfg);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes, 256); return o; };
  L->slices = (int)((T + DWG_SLICE - 1) / DWG_SLICE);
  L->probs = take(T * E * 4);
  L->idx = take(T * k * 4);
  L->w = take(T * k * 4);
  L->d_w = take(T * k * 4);
  L->d_z = take(T * E * 4);
  L->frac = take(E * 4);
  L->xd = take(R * d * 2);
  L->d_yd = take(R * d * 2);
  L->d_xd = take(R * d * 2);
  L->yd = take(gemm2_can_combine(cfg) ? R * d * 2 + 256 : 0);  // (+ counters of the product that recomputes it)
  L->partial = take((size_t)L->slices * d * E * 4);
  L->ffn = take(moe_expert_ffn_backward_workspace_bytes(cfg));
  L->total = off;
}

template <int EC>
int32_t gate_products(const moe_config* cfg, const void* x, const float* w_router, const int32_t* a2r, const float* d_z,
                      const void* d_xd, const void* extra, void* d_x, float* d_w_router, float* partial, int slices,
                      hipStream_t s) {
  const int T = cfg->T, d = cfg->d_model, E = cfg->E;
  const dim3 block(256);
  const unsigned col_blocks = (unsigned)((d / 2 + 255) / 256);
  hipLaunchKernelGGL(dx_kernel<EC>, dim3(col_blocks, (unsigned)((T + GB_TOK - 1) / GB_TOK)), block, 0, s, (const uint32_t*)d_xd, a2r, d_z,
                     w_router, (const uint32_t*)extra, (uint32_t*)d_x, T, d, E, cfg->k);
  hipLaunchKernelGGL(dwg_partial_kernel<EC>, dim3(col_blocks, (unsigned)slices, (unsigned)((E + EC - 1) / EC)), block, 0, s, (const uint32_t*)x, d_z, partial, T, d, E,
                     DWG_SLICE);
  const size_t n = (size_t)d * E;
  hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((n + 255) / 256)), block, 0, s, partial, d_w_router, n, slices);
  return check_hip(hipGetLastError(), "gate backward launch");
}

}  // namespace

extern "C" size_t moe_layer_backward_workspace_bytes(const moe_config* cfg) {
  if (moe_config_check(cfg) != MOE_OK) return 0;
  BwLayout L;
  bw_layout(cfg, &L);
  return L.total;
}

extern "C" int32_t moe_layer_backward(const moe_config* cfg, const moe_weights* w, const void* w1_input_major,
                                      const void* w2_input_major, const void* x, const void* d_out, const void* add_to_d_x,
                                      float aux_loss_coef, const void* fwd_ws, size_t fwd_ws_bytes, void* d_x, float* d_w_router,
                                      float* d_b_router, void* d_w1, float* d_b1, void* d_w2, float* d_b2,
                                      int32_t d_w_dtype, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if ((st = check_weights(cfg, w)) != MOE_OK) return st;
  if (cfg->dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "moe_layer_backward: bf16 only");
  if ((cfg->T + GB_TOK - 1) / GB_TOK > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_layer_backward: at most %d tokens", 65535 * GB_TOK);
  if (!w->w_router || !d_w_router || (w->b_router && !d_b_router))
    return fail(MOE_ERR_INVALID_ARG, "moe_layer_backward: router weights and their gradient buffers must be non-NULL");
  if (cfg->T > 0 && (!x || !d_out || !d_x)) return fail(MOE_ERR_INVALID_ARG, "moe_layer_backward: x, d_out and d_x must be non-NULL");
  moe_ws_layout F;
  moe_workspace_layout(cfg, &F);
  if (!fwd_ws || ((uintptr_t)fwd_ws & 255) || fwd_ws_bytes < F.total)
    return fail(MOE_ERR_WORKSPACE, "moe_layer_backward: the forward workspace has %zu bytes (got %zu)", F.total, fwd_ws_bytes);
  BwLayout L;
  bw_layout(cfg, &L);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < L.total)
    return fail(MOE_ERR_WORKSPACE, "moe_layer_backward: workspace needs %zu bytes, 256-byte aligned (got %zu)", L.total, ws_bytes);
  hipStream_t s = (hipStream_t)stream;
  const char* fb = (const char*)fwd_ws;
  char* b = (char*)ws;
  const float* topk_w = (const float*)(fb + F.topk_w);
  const int32_t* topk_idx = (const int32_t*)(fb + F.topk_idx);
  const int32_t* offsets = (const int32_t*)(fb + F.expert_offsets);
  const int32_t* a2r = (const int32_t*)(fb + F.assign_to_row);
  const void* h = fb + F.h;
  const void* yd = fb + F.yd;
  float* probs = (float*)(b + L.probs);
  float* d_w = (float*)(b + L.d_w);
  float* d_z = (float*)(b + L.d_z);
  if (cfg->T == 0) {  // nothing flows back; the gradients of the parameters are zero
    if ((st = ffn_backward_impl("moe_layer_backward", cfg, w, w1_input_major, w2_input_major, nullptr, nullptr, nullptr, offsets,
                                nullptr, d_w1, d_b1, d_w2, d_b2, d_w_dtype, b + L.ffn, ws_bytes - L.ffn, stream)) != MOE_OK) return st;
    const size_t n = (size_t)cfg->d_model * cfg->E;  // (sums over no slice and no token: zeros)
    hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)(b + L.partial), d_w_router, n, 0);
    if (d_b_router) hipLaunchKernelGGL(gate_dbias_kernel, dim3(cfg->E), dim3(256), 0, s, d_z, d_b_router, 0, cfg->E);
    return check_hip(hipGetLastError(), "moe_layer_backward");
  }
  // the probabilities are not kept by the forward pass: run the gate again (same routing, bit for bit)
  if ((st = launch_gate_of(cfg, w, x, (int32_t*)(b + L.idx), (float*)(b + L.w), probs, s)) != MOE_OK) return st;
  if (gemm2_can_combine(cfg)) {
    // with one expert per token the forward pass wrote `out` directly: recompute the experts' outputs
    int32_t* ctr = (int32_t*)(b + L.yd + align_up((size_t)max_rows(cfg) * cfg->d_model * 2, 256));
    hipLaunchKernelGGL(clear_counters_kernel, dim3(1), dim3(64), 0, s, ctr, 8);
    if ((st = check_hip(hipGetLastError(), "counter clear launch")) != MOE_OK) return st;
    const bool sw = cfg->act == MOE_ACT_SWIGLU;
    if ((st = launch_grouped_matmul_bf16(cfg, h, sw ? w->w_down : w->w2, sw ? nullptr : w->b2, offsets, b + L.yd, cfg->d_model,
                                         cfg->d_ff, ctr, s)) != MOE_OK) return st;
    yd = b + L.yd;
  }
  if ((st = moe_combine_backward(cfg, d_out, yd, a2r, topk_w, b + L.d_yd, d_w, stream)) != MOE_OK) return st;
  if ((st = launch_gather_rows(cfg, x, a2r, b + L.xd, s)) != MOE_OK) return st;
  if ((st = ffn_backward_impl("moe_layer_backward", cfg, w, w1_input_major, w2_input_major, b + L.xd, h, b + L.d_yd, offsets,
                              b + L.d_xd, d_w1, d_b1, d_w2, d_b2, d_w_dtype, b + L.ffn, ws_bytes - L.ffn, stream)) != MOE_OK) return st;
  const float* frac = nullptr;
  if (aux_loss_coef != 0.f) {
    frac = (const float*)(b + L.frac);
    hipLaunchKernelGGL(first_choice_fraction_kernel, dim3(cfg->E), dim3(256), 0, s, topk_idx, (const float*)nullptr, (float*)(b + L.frac),
                       (float*)nullptr, cfg->T, cfg->E, cfg->k);
  }
  hipLaunchKernelGGL(gate_dlogits_kernel, dim3((cfg->T + 3) / 4), dim3(256), 0, s, probs, topk_idx, topk_w, d_w, d_z, cfg->T, cfg->E,
                     cfg->k, cfg->renormalize, frac, aux_loss_coef * (float)cfg->E / (float)cfg->T);
  if (d_b_router) hipLaunchKernelGGL(gate_dbias_kernel, dim3(cfg->E), dim3(256), 0, s, d_z, d_b_router, cfg->T, cfg->E);
  if ((st = check_hip(hipGetLastError(), "gate backward launch")) != MOE_OK) return st;
  float* partial = (float*)(b + L.partial);
  if (cfg->E <= 16)
    return gate_products<16>(cfg, x, w->w_router, a2r, d_z, b + L.d_xd, add_to_d_x, d_x, d_w_router, partial, L.slices, s);
  if (cfg->E <= 32)
    return gate_products<32>(cfg, x, w->w_router, a2r, d_z, b + L.d_xd, add_to_d_x, d_x, d_w_router, partial, L.slices, s);
  return gate_products<64>(cfg, x, w->w_router, a2r, d_z, b + L.d_xd, add_to_d_x, d_x, d_w_router, partial, L.slices, s);
}
