// Expert FFN entry point, the float32 grouped GEMM (correctness configuration)
// and the one-time expert weight transpose.
//
// The bf16 MFMA grouped GEMM lives in grouped_gemm_bf16.hip; the float32 path
// below is a plain LDS-tiled FMA kernel used by the small all-fp32 case, where
// launch latency, not arithmetic, sets the time.
#include "moesys_internal.h"

namespace moesys {

int32_t launch_gemm1_bf16(const moe_config*, const moe_weights*, const void*, const int32_t*, void*, const int32_t*, int32_t*,
                          hipStream_t);
int32_t launch_gemm2_bf16(const moe_config*, const moe_weights*, const void*, const int32_t*, void*, int32_t*, hipStream_t);
int32_t launch_gemm2_combine_bf16(const moe_config*, const moe_weights*, const void*, const int32_t*, const int32_t*,
                                  const float*, const void*, void*, int32_t*, hipStream_t);

namespace {

constexpr int FT = 64;   // tile edge (tokens and features)
constexpr int FK = 16;   // K step

enum { F_GELU = 0, F_SWIGLU = 1, F_BIAS = 2 };

__device__ __forceinline__ float gelu_exact(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_exact(float u) { return u / (1.f + expf(-u)); }

// out[r, n] = epi(sum_k act[r,k] * W_e(n,k) (+ bias)), W_e(n,k) = w[e*N*K + n*sn + k*sk].
template <int EPI>
__global__ __launch_bounds__(256) void ffn_f32_kernel(const float* __restrict__ act, const float* __restrict__ wa,
                                                      const float* __restrict__ wb, const float* __restrict__ bias,
                                                      const int32_t* __restrict__ offsets, float* __restrict__ out,
                                                      int E, int N, int K, long sn, long sk) {
  __shared__ float As[FK][FT + 4];
  __shared__ float Ba[FK][FT + 4];
  __shared__ float Bb[EPI == F_SWIGLU ? FK : 1][FT + 4];
  const int e = blockIdx.z;
  const int row0 = offsets[e] + blockIdx.x * FT;
  const int rows = min(FT, offsets[e + 1] - row0);
  if (rows <= 0) return;
  const int n0 = blockIdx.y * FT;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {}, accb[4][4] = {};
  const float* wae = wa + (size_t)e * N * K;
  const float* wbe = EPI == F_SWIGLU ? wb + (size_t)e * N * K : nullptr;
  for (int k0 = 0; k0 < K; k0 += FK) {
    for (int i = threadIdx.x; i < FT * FK; i += 256) {
      const int r = i / FK, kk = i % FK;
      As[kk][r] = act[(size_t)(row0 + min(r, rows - 1)) * K + k0 + kk];
      const int n = min(n0 + r, N - 1);
      Ba[kk][r] = wae[(size_t)n * sn + (size_t)(k0 + kk) * sk];
      if (EPI == F_SWIGLU) Bb[kk][r] = wbe[(size_t)n * sn + (size_t)(k0 + kk) * sk];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < FK; ++kk) {
      float a[4], b[4], bb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Ba[kk][tx * 4 + i]; }
      if (EPI == F_SWIGLU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) bb[i] = Bb[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if (EPI == F_SWIGLU) accb[i][j] = fmaf(a[i], bb[j], accb[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ty * 4 + i;
    if (r >= rows) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float u = acc[i][j];
      if (EPI == F_SWIGLU) u = silu_exact(u) * accb[i][j];
      else {
        if (bias) u += bias[(size_t)e * N + n];
        if (EPI == F_GELU) u = gelu_exact(u);
      }
      out[(size_t)(row0 + r) * N + n] = u;
    }
  }
}

int32_t launch_f32(const moe_config* cfg, int epi, const float* act, const float* wa, const float* wb,
                   const float* bias, const int32_t* offsets, float* out, int N, int K, int layout, hipStream_t s) {
  const int64_t rmax = max_rows(cfg);
  if (rmax == 0) return MOE_OK;
  int64_t per_expert = rmax;  // one expert may hold every row
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS && C < per_expert) per_expert = C;
  dim3 grid((unsigned)((per_expert + FT - 1) / FT), (unsigned)((N + FT - 1) / FT), (unsigned)cfg->E), block(256);
  if (grid.x > 65535u * 32u) return fail(MOE_ERR_UNSUPPORTED, "float32 FFN: too many row tiles");
  const long sn = layout == MOE_LAYOUT_OUTPUT_MAJOR ? K : 1, sk = layout == MOE_LAYOUT_OUTPUT_MAJOR ? 1 : N;
  if (epi == F_GELU) hipLaunchKernelGGL(ffn_f32_kernel<F_GELU>, grid, block, 0, s, act, wa, wb, bias, offsets, out, cfg->E, N, K, sn, sk);
  else if (epi == F_SWIGLU) hipLaunchKernelGGL(ffn_f32_kernel<F_SWIGLU>, grid, block, 0, s, act, wa, wb, bias, offsets, out, cfg->E, N, K, sn, sk);
  else hipLaunchKernelGGL(ffn_f32_kernel<F_BIAS>, grid, block, 0, s, act, wa, wb, bias, offsets, out, cfg->E, N, K, sn, sk);
  return check_hip(hipGetLastError(), "float32 FFN launch");
}

template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows, int cols) {
  __shared__ T tile[32][33];
  const size_t base = (size_t)blockIdx.z * rows * cols;
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < 32; i += 8)
    if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[base + (size_t)(r0 + i) * cols + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 32; i += 8)
    if (c0 + i < cols && r0 + tx < rows) dst[base + (size_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

__global__ void clear_ints_kernel(int32_t* p, int n) {
  if ((int)threadIdx.x < n) p[threadIdx.x] = 0;
}

}  // namespace

int32_t launch_gemm1(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets, void* h,
                     const int32_t* row_map, int32_t* tile_counters, hipStream_t s) {
  if (cfg->dtype == MOE_BF16) return launch_gemm1_bf16(cfg, w, xd, offsets, h, row_map, tile_counters, s);
  if (row_map) return fail(MOE_ERR_UNSUPPORTED, "float32 FFN reads dispatched rows only");
  if (cfg->act == MOE_ACT_SWIGLU)
    return launch_f32(cfg, F_SWIGLU, (const float*)xd, (const float*)w->w_gate_proj, (const float*)w->w_up, nullptr,
                      offsets, (float*)h, cfg->d_ff, cfg->d_model, w->layout, s);
  return launch_f32(cfg, F_GELU, (const float*)xd, (const float*)w->w1, nullptr, (const float*)w->b1, offsets,
                    (float*)h, cfg->d_ff, cfg->d_model, w->layout, s);
}

int32_t launch_gemm2(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets, void* yd,
                     int32_t* tile_counters, hipStream_t s) {
  if (cfg->dtype == MOE_BF16) return launch_gemm2_bf16(cfg, w, h, offsets, yd, tile_counters, s);
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  return launch_f32(cfg, F_BIAS, (const float*)h, (const float*)(sw ? w->w_down : w->w2), nullptr,
                    (const float*)(sw ? nullptr : w->b2), offsets, (float*)yd, cfg->d_model, cfg->d_ff, w->layout, s);
}

// With one expert per token a dispatched row is the only term of its token's output, so the second GEMM can
// finish the combine itself (bf16 only).
bool gemm2_can_combine(const moe_config* cfg) { return cfg->dtype == MOE_BF16 && cfg->k == 1; }

int32_t launch_gemm2_combine(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                             const int32_t* r2a, const float* topk_w, const void* residual, void* out,
                             int32_t* tile_counters, hipStream_t s) {
  if (!gemm2_can_combine(cfg)) return fail(MOE_ERR_UNSUPPORTED, "combine in the second GEMM needs bf16 and k = 1");
  return launch_gemm2_combine_bf16(cfg, w, h, offsets, r2a, topk_w, residual, out, tile_counters, s);
}

}  // namespace moesys

using namespace moesys;

extern "C" int32_t moe_expert_ffn(const moe_config* cfg, const moe_weights* w, const void* xd,
                                  const int32_t* expert_offsets, void* yd, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  st = check_weights(cfg, w);
  if (st != MOE_OK) return st;
  if (!expert_offsets) return fail(MOE_ERR_INVALID_ARG, "moe_expert_ffn: expert_offsets is NULL");
  const size_t need = moe_workspace_bytes(cfg, MOE_WS_FFN);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(MOE_ERR_WORKSPACE, "moe_expert_ffn: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, ws_bytes);
  if (max_rows(cfg) > 0 && (!xd || !yd)) return fail(MOE_ERR_INVALID_ARG, "moe_expert_ffn: xd and yd must be non-NULL");
  // the tile counters sit behind h; nothing ran before us on this workspace, so clear the first GEMM's here
  int32_t* ctr = (int32_t*)((char*)ws + ffn_counter_offset(cfg));
  if (cfg->dtype == MOE_BF16) {
    hipLaunchKernelGGL(clear_ints_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, ctr, 8);
    if ((st = check_hip(hipGetLastError(), "counter clear launch")) != MOE_OK) return st;
  }
  st = launch_gemm1(cfg, w, xd, expert_offsets, ws, nullptr, ctr, (hipStream_t)stream);
  if (st != MOE_OK) return st;
  return launch_gemm2(cfg, w, ws, expert_offsets, yd, ctr, (hipStream_t)stream);
}

extern "C" int32_t moe_transpose_expert_weights(const void* src, void* dst, int32_t E, int32_t rows, int32_t cols,
                                                int32_t dtype, void* stream) {
  if (!src || !dst || src == dst) return fail(MOE_ERR_INVALID_ARG, "moe_transpose_expert_weights: src/dst NULL or aliased");
  if (E < 1 || rows < 1 || cols < 1 || E > 65535) return fail(MOE_ERR_INVALID_ARG, "moe_transpose_expert_weights: bad shape");
  if (dtype != MOE_F32 && dtype != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "moe_transpose_expert_weights: dtype unknown");
  dim3 grid((cols + 31) / 32, (rows + 31) / 32, E), block(256);
  if (grid.y > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_transpose_expert_weights: rows too large");
  if (dtype == MOE_BF16)
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, block, 0, (hipStream_t)stream, (const uint16_t*)src, (uint16_t*)dst, rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, block, 0, (hipStream_t)stream, (const float*)src, (float*)dst, rows, cols);
  return check_hip(hipGetLastError(), "transpose launch");
}
