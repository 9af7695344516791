// Expert FFN products for steps of very few tokens (k*T <= 16 assignments in all, so no expert has more rows
// than that): the single-request end of the paper's inference scenario (Section 3.3, batch size 1).
//
//   out[r, n] = epilogue( sum_k act[r, k] * W_e[n, k] )      for the rows r of every expert e that has any
//
// With one or two rows per activated expert the product is a matrix-vector product: its time is the time to
// stream the activated experts' weights once, and the MFMA tiles of the grouped GEMM (256 output features per
// workgroup) leave most CUs without work: 2 experts x N/256 tiles.  Here a wavefront owns FPW weight rows
// and its 64 lanes split the contraction index (16 bytes per lane and row: every weight row is read with
// wave-wide contiguous 1 KB loads, FPW of them in flight per wavefront and K block), keeps the partial sums
// of its weight rows x the expert's rows in registers, and adds them across the lanes at the end (a fixed
// butterfly: results do not depend on scheduling).  Workgroup (bx, r0) serves the expert whose FIRST row is
// dispatched row r0 and exits if there is none, so the grid needs no list of the activated experts.  Two shapes
// (the FPW x ROWS partial sums must fit the registers): 8 weight rows x up to 8 rows, 4 x up to 16.
#include "moesys_internal.h"

namespace moesys {
namespace {

constexpr int GV_MAX_ROWS = 16;  // rows of one expert, at most (= assignments of the whole step)
constexpr int GV_WAVES = 4;

enum GvEpi { GV_GELU = 0, GV_SWIGLU = 1, GV_BIAS = 2, GV_COMBINE = 3 };

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint16_t bf16_of(float v) {  // round to nearest even
  return (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{v, 0.f}, bf16x2)) & 0xffffu);
}
__device__ __forceinline__ float gelu_exact(float u) { return 0.5f * u * erfcf(-u * 0.70710678118654752f); }

// EPI: GV_GELU out = gelu(. + bias); GV_SWIGLU out = silu(. Wg) * (. Wu) (a wavefront's weight rows are
// FPW/2 of Wg and the same FPW/2 of Wu); GV_BIAS out = . + bias; GV_COMBINE (k = 1) out[token] =
// residual[token] + gate_w[token] * (. + bias) with token = row_map[r].
// GATHER: act is x[T, K] and row r reads token row_map[r] mod T.
// KSPLIT: the four wavefronts of a workgroup share one set of GV_FPW weight rows and split the contraction index
// (their sums meet in LDS, in wavefront order): four times the workgroups, for long rows and few experts.
template <int EPI, bool GATHER, int GV_ROWS, int GV_FPW, bool KSPLIT>
__global__ __launch_bounds__(GV_WAVES * 64) void expert_gemv_kernel(
    const uint16_t* __restrict__ act, const uint16_t* __restrict__ wa, const uint16_t* __restrict__ wb,
    const uint16_t* __restrict__ bias, const int32_t* __restrict__ offsets, uint16_t* out,
    const int32_t* __restrict__ row_map, const float* __restrict__ gate_w, const uint16_t* residual,
    const int64_t* __restrict__ eoff, int T, int E, int N, int K, int reps) {
  constexpr int OUTF = EPI == GV_SWIGLU ? GV_FPW / 2 : GV_FPW;  // output features per wavefront
  __shared__ int s_e;
  __shared__ float red[KSPLIT ? GV_WAVES : 1][GV_ROWS][GV_FPW];
  const int r0 = blockIdx.y;
  if (threadIdx.x == 0) s_e = -1;
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += GV_WAVES * 64)
    if (offsets[e] == r0 && offsets[e + 1] > r0) s_e = e;  // at most one expert starts at row r0
  __syncthreads();
  const int e = s_e;
  if (e < 0) return;
  const int rows = min(offsets[e + 1] - r0, GV_ROWS);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t wbase = eoff ? eoff[e] : (int64_t)e * N * K;
  const uint16_t* xrow[GV_ROWS];
  int token[GV_ROWS];
#pragma unroll
  for (int r = 0; r < GV_ROWS; ++r) {
    const int rr = r0 + min(r, rows - 1);  // (rows past the expert's last re-read it; their sums are not used)
    int src = rr;
    token[r] = 0;
    if (GATHER || EPI == GV_COMBINE) {
      int t = row_map[rr];
      while (t >= T) t -= T;  // assignment id j*T + t -> token (j < k <= 8)
      token[r] = t;
      if (GATHER) src = t;
    }
    xrow[r] = act + (int64_t)src * K;
  }

  // a workgroup works through `reps` consecutive blocks of output features (with a short contraction index one
  // block is too little work per workgroup)
  for (int rep = 0; rep < reps; ++rep) {
    // first output feature of this wavefront
    const int n0 = KSPLIT ? (blockIdx.x * reps + rep) * OUTF : ((blockIdx.x * reps + rep) * GV_WAVES + wave) * OUTF;
    const uint16_t* wrow[GV_FPW];
#pragma unroll
    for (int j = 0; j < GV_FPW; ++j) {
      if (EPI == GV_SWIGLU) wrow[j] = (j < OUTF ? wa : wb) + wbase + (int64_t)(n0 + j % OUTF) * K;
      else wrow[j] = wa + wbase + (int64_t)(n0 + j) * K;
    }
    float acc[GV_FPW][GV_ROWS];
  #pragma unroll
    for (int j = 0; j < GV_FPW; ++j)
  #pragma unroll
      for (int r = 0; r < GV_ROWS; ++r) acc[j][r] = 0.f;

    for (int kb = (KSPLIT ? (int)threadIdx.x : lane) * 8; kb < K; kb += (KSPLIT ? GV_WAVES : 1) * 64 * 8) {
      uint4 wv[GV_FPW], xv[GV_ROWS];
  #pragma unroll
      for (int j = 0; j < GV_FPW; ++j) wv[j] = *reinterpret_cast<const uint4*>(wrow[j] + kb);
  #pragma unroll
      for (int r = 0; r < GV_ROWS; ++r)
        if (r < rows) xv[r] = *reinterpret_cast<const uint4*>(xrow[r] + kb);
  #pragma unroll
      for (int r = 0; r < GV_ROWS; ++r) {
        if (r < rows) {  // (wave-uniform)
          const float x0 = lo16(xv[r].x), x1 = hi16(xv[r].x), x2 = lo16(xv[r].y), x3 = hi16(xv[r].y);
          const float x4 = lo16(xv[r].z), x5 = hi16(xv[r].z), x6 = lo16(xv[r].w), x7 = hi16(xv[r].w);
  #pragma unroll
          for (int j = 0; j < GV_FPW; ++j) {
            float a = acc[j][r];
            a = fmaf(lo16(wv[j].x), x0, a); a = fmaf(hi16(wv[j].x), x1, a);
            a = fmaf(lo16(wv[j].y), x2, a); a = fmaf(hi16(wv[j].y), x3, a);
            a = fmaf(lo16(wv[j].z), x4, a); a = fmaf(hi16(wv[j].z), x5, a);
            a = fmaf(lo16(wv[j].w), x6, a); a = fmaf(hi16(wv[j].w), x7, a);
            acc[j][r] = a;
          }
        }
      }
    }

    // sums over the lanes; afterwards every lane holds every total
  #pragma unroll
    for (int r = 0; r < GV_ROWS; ++r) {
      if (r < rows) {
  #pragma unroll
        for (int j = 0; j < GV_FPW; ++j) {
          float v = acc[j][r];
  #pragma unroll
          for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
          acc[j][r] = v;
        }
      }
    }

    if constexpr (KSPLIT) {  // the wavefronts' sums meet: lane j < GV_FPW carries weight row j
      if (rep) __syncthreads();  // (the previous block's sums have been read)
#pragma unroll
      for (int r = 0; r < GV_ROWS; ++r) {
        if (r < rows && lane < GV_FPW) {
          float v = acc[0][r];
#pragma unroll
          for (int j = 1; j < GV_FPW; ++j) v = lane == j ? acc[j][r] : v;
          red[wave][r][lane] = v;
        }
      }
      __syncthreads();
      if (wave == 0 && lane < GV_FPW) {
#pragma unroll
        for (int r = 0; r < GV_ROWS; ++r) {
          if (r < rows) {
            float v = red[0][r][lane];
#pragma unroll
            for (int w = 1; w < GV_WAVES; ++w) v += red[w][r][lane];
            red[0][r][lane] = v;  // (only this lane reads and writes the element)
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int r = 0; r < GV_ROWS; ++r)
        if (r < rows)
#pragma unroll
          for (int j = 0; j < GV_FPW; ++j) acc[j][r] = red[0][r][j];  // every lane holds every total again
    }
    // lane j < OUTF finishes output feature n0 + j of every row
    if ((!KSPLIT || wave == 0) && lane < OUTF) {
      const int n = n0 + lane;
      float b = 0.f;
      if (EPI != GV_SWIGLU && bias) b = lo16((uint32_t)bias[(eoff ? eoff[e] : (int64_t)e * N) + n]);  // (eoff: as for the weights)
  #pragma unroll
      for (int r = 0; r < GV_ROWS; ++r) {
        if (r < rows) {
          float v = acc[0][r], u = 0.f;
  #pragma unroll
          for (int j = 1; j < OUTF; ++j) v = lane == j ? acc[j][r] : v;
          if (EPI == GV_SWIGLU) {
            u = acc[OUTF][r];
  #pragma unroll
            for (int j = 1; j < OUTF; ++j) u = lane == j ? acc[OUTF + j][r] : u;
            v = v * __builtin_amdgcn_rcpf(1.f + __expf(-v)) * u;
          } else {
            v += b;
            if (EPI == GV_GELU) v = gelu_exact(v);
          }
          if (EPI == GV_COMBINE) {
            const size_t o = (size_t)token[r] * N + n;
            const float res = residual ? lo16((uint32_t)residual[o]) : 0.f;
            out[o] = bf16_of(fmaf(gate_w[token[r]], v, res));
          } else {
            out[(size_t)(r0 + r) * N + n] = bf16_of(v);
          }
        }
      }
    }
  }
}

// A step of ONE token with k >= 2 experts: the second product and the combine in one kernel.  A workgroup owns
// C1_FPW output features; for the k choices in turn (row = assign_to_row[j], its expert from the offsets table)
// its four wavefronts split the contraction index, the sums meet in LDS in wavefront order, the result (+ bias)
// is rounded to bf16 and stored in yd as the separate product would store it, and out accumulates
// residual + sum_j w_j * yd[row_j] from those rounded values, in float32 and in the order of the combine kernel.
constexpr int C1_FPW = 8;

__global__ __launch_bounds__(GV_WAVES * 64) void expert_gemv_combine1_kernel(
    const uint16_t* __restrict__ h, const uint16_t* __restrict__ w2, const uint16_t* __restrict__ bias,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ a2r, const float* __restrict__ topk_w,
    const uint16_t* residual, uint16_t* __restrict__ yd, uint16_t* out, const int64_t* __restrict__ eoff, int E, int N,
    int K, int k) {
  __shared__ int s_e[MOE_MAX_TOPK];  // expert of dispatched row r (T = 1: there are exactly k rows)
  __shared__ float red[GV_WAVES][C1_FPW];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (int e = threadIdx.x; e < E; e += GV_WAVES * 64)
    for (int r = offsets[e]; r < offsets[e + 1] && r < MOE_MAX_TOPK; ++r) s_e[r] = e;
  __syncthreads();
  const int n0 = blockIdx.x * C1_FPW;
  float o = 0.f;  // (used by lanes < C1_FPW of wavefront 0: output feature n0 + lane)
  if (wave == 0 && lane < C1_FPW && residual) o = lo16((uint32_t)residual[n0 + lane]);
  for (int j = 0; j < k; ++j) {
    const int row = a2r[j];
    if (row < 0) continue;  // (cannot happen with one token: the capacity is at least one; uniform anyway)
    const int e = s_e[row];
    const uint16_t* wbase = w2 + (eoff ? eoff[e] : (int64_t)e * N * K) + (int64_t)n0 * K;
    const uint16_t* xrow = h + (int64_t)row * K;
    float acc[C1_FPW];
#pragma unroll
    for (int f = 0; f < C1_FPW; ++f) acc[f] = 0.f;
#pragma unroll 2
    for (int kb = (int)threadIdx.x * 8; kb < K; kb += GV_WAVES * 64 * 8) {
      uint4 wv[C1_FPW];
#pragma unroll
      for (int f = 0; f < C1_FPW; ++f) wv[f] = *reinterpret_cast<const uint4*>(wbase + (int64_t)f * K + kb);
      const uint4 xv = *reinterpret_cast<const uint4*>(xrow + kb);
      const float x0 = lo16(xv.x), x1 = hi16(xv.x), x2 = lo16(xv.y), x3 = hi16(xv.y);
      const float x4 = lo16(xv.z), x5 = hi16(xv.z), x6 = lo16(xv.w), x7 = hi16(xv.w);
#pragma unroll
      for (int f = 0; f < C1_FPW; ++f) {
        float a = acc[f];
        a = fmaf(lo16(wv[f].x), x0, a); a = fmaf(hi16(wv[f].x), x1, a);
        a = fmaf(lo16(wv[f].y), x2, a); a = fmaf(hi16(wv[f].y), x3, a);
        a = fmaf(lo16(wv[f].z), x4, a); a = fmaf(hi16(wv[f].z), x5, a);
        a = fmaf(lo16(wv[f].w), x6, a); a = fmaf(hi16(wv[f].w), x7, a);
        acc[f] = a;
      }
    }
    float mine = 0.f;  // lane f < C1_FPW: the wavefront's sum for output feature n0 + f
#pragma unroll
    for (int f = 0; f < C1_FPW; ++f) {
      float v = acc[f];
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
      mine = lane == f ? v : mine;
    }
    if (lane < C1_FPW) red[wave][lane] = mine;
    __syncthreads();
    if (wave == 0 && lane < C1_FPW) {
      float v = red[0][lane];
#pragma unroll
      for (int w = 1; w < GV_WAVES; ++w) v += red[w][lane];
      if (bias) v += lo16((uint32_t)bias[(eoff ? eoff[e] : (int64_t)e * N) + n0 + lane]);
      const uint16_t yb = bf16_of(v);
      yd[(size_t)row * N + n0 + lane] = yb;
      o = fmaf(topk_w[j], lo16((uint32_t)yb), o);
    }
    __syncthreads();  // (red is free for the next choice)
  }
  if (wave == 0 && lane < C1_FPW) out[n0 + lane] = bf16_of(o);
}

template <int EPI, int ROWS, int FPW>
int32_t launch_shape(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb, const uint16_t* bias,
                     const int32_t* offsets, uint16_t* out, const int32_t* row_map, const float* gate_w, const uint16_t* residual,
                     const int64_t* eoff, int N, int K, bool gather, hipStream_t s) {
  constexpr int OUTF = EPI == GV_SWIGLU ? FPW / 2 : FPW;
  // About 256 KB of weights per workgroup, in whole blocks of output features, as long as that leaves about two
  // workgroups per CU (the experts with rows are at most k*T).  Long rows and too few workgroups even so: the
  // wavefronts of a workgroup split the contraction index instead of the output features.
  const int A = cfg->k * cfg->T;
  int blocks = N / (GV_WAVES * OUTF);
  const bool ksplit = K >= 4096 && (int64_t)blocks * A < 512;
  if (ksplit) blocks *= GV_WAVES;
  int reps = ksplit ? 1 : (int)((256 * 1024) / ((int64_t)GV_WAVES * FPW * K * 2));
  reps = reps < 1 ? 1 : reps > 8 ? 8 : reps;
  while (reps > 1 && (blocks % reps || (int64_t)(blocks / reps) * A < 512)) --reps;
  const dim3 grid(blocks / reps, A), block(GV_WAVES * 64);
#define MOESYS_GEMV(G, S)                                                                                                  \
  hipLaunchKernelGGL((expert_gemv_kernel<EPI, G, ROWS, FPW, S>), grid, block, 0, s, act, wa, wb, bias, offsets, out, row_map, \
                     gate_w, residual, eoff, cfg->T, cfg->E, N, K, reps)
  if (gather) { if (ksplit) MOESYS_GEMV(true, true); else MOESYS_GEMV(true, false); }
  else { if (ksplit) MOESYS_GEMV(false, true); else MOESYS_GEMV(false, false); }
#undef MOESYS_GEMV
  return check_hip(hipGetLastError(), "expert GEMV launch");
}

template <int EPI>
int32_t launch(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb, const uint16_t* bias,
               const int32_t* offsets, uint16_t* out, const int32_t* row_map, const float* gate_w, const uint16_t* residual,
               const int64_t* eoff, int N, int K, bool gather, hipStream_t s) {
  const int A = cfg->k * cfg->T;
  if (A == 0) return MOE_OK;
  if (A <= 8) return launch_shape<EPI, 8, 8>(cfg, act, wa, wb, bias, offsets, out, row_map, gate_w, residual, eoff, N, K, gather, s);
  return launch_shape<EPI, 16, 4>(cfg, act, wa, wb, bias, offsets, out, row_map, gate_w, residual, eoff, N, K, gather, s);
}

}  // namespace

// Whether the few-row path serves this product: so few assignments that no expert exceeds GV_MAX_ROWS rows,
// whole workgroups of output features, 16-byte chunks of the contraction index.
bool expert_gemv_applies(const moe_config* cfg, int N, int K) {
  return tuning(MOE_TUNE_FEW_TOKEN_KERNELS) != 0 && cfg->dtype == MOE_BF16 && (int64_t)cfg->k * cfg->T <= GV_MAX_ROWS && N % (GV_WAVES * 8) == 0 && K % 8 == 0;
}

// Second product + combine of a one-token step (k >= 2); see the kernel.  residual nullable; out may be residual.
bool expert_gemv_combine_one_token_applies(const moe_config* cfg) {
  return cfg->T == 1 && cfg->k >= 2 && expert_gemv_applies(cfg, cfg->d_model, cfg->d_ff);
}
int32_t launch_expert_gemv_combine_one_token(const moe_config* cfg, const void* h, const void* w2, const void* bias,
                                             const int32_t* offsets, const int32_t* a2r, const float* topk_w,
                                             const void* residual, void* yd, void* out, const int64_t* eoff, hipStream_t s) {
  if (!expert_gemv_combine_one_token_applies(cfg)) return fail(MOE_ERR_UNSUPPORTED, "expert GEMV: not a one-token step");
  hipLaunchKernelGGL(expert_gemv_combine1_kernel, dim3(cfg->d_model / C1_FPW), dim3(GV_WAVES * 64), 0, s, (const uint16_t*)h,
                     (const uint16_t*)w2, (const uint16_t*)bias, offsets, a2r, topk_w, (const uint16_t*)residual, (uint16_t*)yd,
                     (uint16_t*)out, eoff, cfg->E, cfg->d_model, cfg->d_ff, cfg->k);
  return check_hip(hipGetLastError(), "expert GEMV launch");
}

// epi: 0 GELU (+bias), 1 SwiGLU (wa = gate, wb = up), 2 plain (+bias), 3 combine for k = 1 (row_map = row_to_assign,
// gate_w, residual).  row_map with epi 0/1: gather the rows from x[T, K].  eoff: per-expert element offsets or NULL.
int32_t launch_expert_gemv_bf16(int epi, const moe_config* cfg, const void* act, const void* wa, const void* wb, const void* bias,
                                const int32_t* offsets, void* out, const int32_t* row_map, const float* gate_w,
                                const void* residual, const int64_t* eoff, int N, int K, hipStream_t s) {
  if (!expert_gemv_applies(cfg, N, K)) return fail(MOE_ERR_UNSUPPORTED, "expert GEMV: shape outside the few-row path");
  const uint16_t *a = (const uint16_t*)act, *w0 = (const uint16_t*)wa, *w1 = (const uint16_t*)wb, *b = (const uint16_t*)bias;
  const uint16_t* res = (const uint16_t*)residual;
  switch (epi) {
    case GV_GELU: return launch<GV_GELU>(cfg, a, w0, w1, b, offsets, (uint16_t*)out, row_map, gate_w, res, eoff, N, K, row_map != nullptr, s);
    case GV_SWIGLU: return launch<GV_SWIGLU>(cfg, a, w0, w1, nullptr, offsets, (uint16_t*)out, row_map, gate_w, res, eoff, N, K, row_map != nullptr, s);
    case GV_BIAS: return launch<GV_BIAS>(cfg, a, w0, w1, b, offsets, (uint16_t*)out, nullptr, gate_w, res, eoff, N, K, false, s);
    case GV_COMBINE:
      if (!row_map || !gate_w || cfg->k != 1) return fail(MOE_ERR_INVALID_ARG, "expert GEMV: combine epilogue needs k = 1, row map and gate weights");
      return launch<GV_COMBINE>(cfg, a, w0, w1, b, offsets, (uint16_t*)out, row_map, gate_w, res, eoff, N, K, false, s);
  }
  return fail(MOE_ERR_INVALID_ARG, "expert GEMV: unknown epilogue");
}

}  // namespace moesys
