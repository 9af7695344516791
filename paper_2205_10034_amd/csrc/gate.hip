// Top-k softmax gate (GShard top-2 / top-1 gating, Section 5.2; softmax in fp32, Section 5.2).
//
// Exact path: one wavefront works on TPW tokens at a time.  Each lane owns a
// strided slice of d_model and accumulates the logits of NE experts in
// float64 (the product of two float32 / bfloat16 values is exact in float64,
// so only the summation rounds, at 2^-53 relative).  A reduce-scatter over the
// 64 lanes leaves one expert's logit per lane group, the logits go through
// LDS, and the wave then does the fp32 softmax and k rounds of arg-max
// (ties -> lower expert index) with cross-lane shuffles.
#include "moesys_internal.h"

namespace moesys {
namespace {

constexpr int NE = 16;   // experts per accumulation pass
constexpr int TPW = 4;   // tokens per wavefront
constexpr int WAVES = 4; // wavefronts per block

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <typename XT> struct XLoad;
template <> struct XLoad<float> {
  static constexpr int V = 4;
  static __device__ __forceinline__ void load(const float* p, float (&o)[4]) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct XLoad<uint16_t> {
  static constexpr int V = 8;
  static __device__ __forceinline__ void load(const uint16_t* p, float (&o)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

__device__ __forceinline__ double shfl_xor_f64(double v, int m) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, m, 64);
  hi = __shfl_xor(hi, m, 64);
  return __hiloint2double(hi, lo);
}

template <int W, int M>
__device__ __forceinline__ void rs_step(double (&acc)[NE], int lane) {
  const bool upper = (lane & M) != 0;
#pragma unroll
  for (int i = 0; i < W; ++i) {
    double send = upper ? acc[i] : acc[i + W];
    double keep = upper ? acc[i + W] : acc[i];
    acc[i] = keep + shfl_xor_f64(send, M);
  }
}

// After the call every lane holds the wave-wide sum of acc[(lane >> 2) & 15].
__device__ __forceinline__ double reduce_scatter16(double (&acc)[NE], int lane) {
  rs_step<8, 32>(acc, lane);
  rs_step<4, 16>(acc, lane);
  rs_step<2, 8>(acc, lane);
  rs_step<1, 4>(acc, lane);
  double v = acc[0];
  v += shfl_xor_f64(v, 2);
  v += shfl_xor_f64(v, 1);
  return v;
}

template <typename XT>
__global__ __launch_bounds__(WAVES * 64) void gate_exact_kernel(
    const XT* __restrict__ x, const float* __restrict__ wr, const float* __restrict__ br, int T, int d,
    int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    float* __restrict__ probs) {
  extern __shared__ double zs_all[];  // [WAVES][TPW][Epad]
  constexpr int V = XLoad<XT>::V;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int Epad = (E + NE - 1) / NE * NE;
  double* zs = zs_all + (size_t)wave * TPW * Epad;
  const int t0 = (blockIdx.x * WAVES + wave) * TPW;

  for (int c0 = 0; c0 < E; c0 += NE) {
    const int ne = min(NE, E - c0);
    double acc[TPW][NE];
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
      for (int e = 0; e < NE; ++e) acc[q][e] = 0.0;
    for (int i = lane * V; i < d; i += 64 * V) {
      float xv[TPW][V];
#pragma unroll
      for (int q = 0; q < TPW; ++q) {
        const int t = min(t0 + q, T - 1);  // clamp: tail tokens recompute the last row, never stored
        XLoad<XT>::load(x + (size_t)t * d + i, xv[q]);
      }
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const float* wrow = wr + (size_t)(i + v) * E + c0;
        float wv[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) wv[e] = e < ne ? wrow[e] : 0.f;
#pragma unroll
        for (int q = 0; q < TPW; ++q)
#pragma unroll
          for (int e = 0; e < NE; ++e) acc[q][e] = fma((double)xv[q][v], (double)wv[e], acc[q][e]);
      }
    }
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
      double z = reduce_scatter16(acc[q], lane);
      const int e = (lane >> 2) & 15;
      if ((lane & 3) == 0 && e < ne) zs[q * Epad + c0 + e] = z + (br ? (double)br[c0 + e] : 0.0);
    }
  }
  __syncthreads();

  for (int q = 0; q < TPW; ++q) {
    const int t = t0 + q;
    if (t >= T) break;  // uniform per wave
    // each lane owns experts lane, lane+64, ...
    double zd[4];
    float zf[4];
    float mx = -INFINITY;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int e = lane + 64 * s;
      zd[s] = e < E ? zs[q * Epad + e] : -INFINITY;
      zf[s] = (float)zd[s];
      mx = fmaxf(mx, zf[s]);
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    float ex[4], sum = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      ex[s] = (lane + 64 * s) < E ? expf(zf[s] - mx) : 0.f;
      sum += ex[s];
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
    float p[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      p[s] = ex[s] / sum;
      if (probs && (lane + 64 * s) < E) probs[(size_t)t * E + lane + 64 * s] = p[s];
    }
    // k rounds of arg-max on the float64 logits; ties -> lower expert index
    float wsel = 0.f, wsum = 0.f;  // lane j keeps the j-th selection
    int isel = 0;
    for (int j = 0; j < k; ++j) {
      double bz = -INFINITY;
      int be = 0x7fffffff;
      float bp = 0.f;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const int e = lane + 64 * s;
        if (e < E && (zd[s] > bz || (zd[s] == bz && e < be))) { bz = zd[s]; be = e; bp = p[s]; }
      }
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) {
        double oz = shfl_xor_f64(bz, m);
        int oe = __shfl_xor(be, m, 64);
        float op = __shfl_xor(bp, m, 64);
        if (oz > bz || (oz == bz && oe < be)) { bz = oz; be = oe; bp = op; }
      }
      // retire the winner (all lanes agree on be)
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (lane + 64 * s == be) zd[s] = -INFINITY;
      if (lane == j) { isel = be; wsel = bp; }
      wsum += bp;
    }
    if (lane < k) {
      topk_idx[(size_t)t * k + lane] = isel;
      topk_w[(size_t)t * k + lane] = renorm ? wsel / wsum : wsel;
    }
  }
}

}  // namespace

int32_t launch_gate(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                    int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  const int per_block = WAVES * TPW;
  dim3 grid((cfg->T + per_block - 1) / per_block), block(WAVES * 64);
  const int Epad = (cfg->E + NE - 1) / NE * NE;
  size_t shmem = (size_t)WAVES * TPW * Epad * sizeof(double);
  if (cfg->dtype == MOE_BF16)
    hipLaunchKernelGGL(gate_exact_kernel<uint16_t>, grid, block, shmem, s, (const uint16_t*)x, w_router,
                       b_router, cfg->T, cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w,
                       probs);
  else
    hipLaunchKernelGGL(gate_exact_kernel<float>, grid, block, shmem, s, (const float*)x, w_router, b_router,
                       cfg->T, cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w, probs);
  return check_hip(hipGetLastError(), "gate launch");
}

}  // namespace moesys

using namespace moesys;

extern "C" int32_t moe_gate(const moe_config* cfg, const void* x, const float* w_router,
                            const float* b_router, int32_t* topk_idx, float* topk_w, float* probs,
                            void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (cfg->T > 0 && (!x || !w_router || !topk_idx || !topk_w))
    return fail(MOE_ERR_INVALID_ARG, "moe_gate: x, w_router, topk_idx and topk_w must be non-NULL");
  return launch_gate(cfg, x, w_router, b_router, topk_idx, topk_w, probs, (hipStream_t)stream);
}
