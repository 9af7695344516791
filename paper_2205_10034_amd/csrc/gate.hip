// Top-k softmax gate (GShard top-2 / top-1 gating, Section 5.2; softmax in fp32, Section 5.2).
//
// Two kernels.
//
// Fast path (bf16 activations, E <= 64), HBM-bound: the logits are a skinny GEMM on the MFMA units.
// Activations are bfloat16 already; every float32 router weight is split into three bfloat16 pieces
// (w = hi + mid + lo exactly), so every product is exact in float32 and the only rounding is the
// accumulation: float32 inside a 64-wide K chunk (24 roundings at most), float64 across chunks and
// across the four wavefronts that share the K range.  The logits therefore carry an error of about
// 1e-7.  Ranking needs more: it must equal the ranking of the exactly computed logits.  Any token whose
// k+1 leading logits have two neighbours closer than GATE_MARGIN_REL times its largest |logit| is recomputed by the whole workgroup
// with float64 accumulation of the (exact) products and ranked on those values.
//
// Exact path (float32 activations, or E > 64): one wavefront works on TPW tokens at a time.  Each lane owns a
// strided slice of d_model and accumulates the logits of NE experts in
// float64 (the product of two float32 / bfloat16 values is exact in float64,
// so only the summation rounds, at 2^-53 relative).  A reduce-scatter over the
// 64 lanes leaves one expert's logit per lane group, the logits go through
// LDS, and the wave then does the fp32 softmax and k rounds of arg-max
// (ties -> lower expert index) with cross-lane shuffles.
#include <type_traits>
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

// A lane's partner inside its group of eight consecutive lanes, for the three steps of a reduction over the group:
// steps 0 and 1 swap lanes inside a quad (lane ^ 1, lane ^ 2), step 2 mirrors the eight lanes (lane i with 7 - i,
// which lies in the other quad).  Data-parallel-primitive moves on the vector ALU: a few clocks each, where a
// general lane permutation goes through the LDS crossbar (a hundred clocks, and a reduction is a chain of them).
template <int STEP>
__device__ __forceinline__ int group8_partner(int v) {
  constexpr int ctrl = STEP == 0 ? 0xB1 /* quad_perm 1,0,3,2 */ : STEP == 1 ? 0x4E /* quad_perm 2,3,0,1 */ : 0x141 /* row_half_mirror */;
  return __builtin_amdgcn_update_dpp(0, v, ctrl, 0xF, 0xF, true);
}
template <int STEP>
__device__ __forceinline__ float group8_partner(float v) { return __int_as_float(group8_partner<STEP>(__float_as_int(v))); }
template <int STEP>
__device__ __forceinline__ double group8_partner(double v) {
  return __hiloint2double(group8_partner<STEP>(__double2hiint(v)), group8_partner<STEP>(__double2loint(v)));
}
// f(step) for the three steps, unrolled
template <typename F>
__device__ __forceinline__ void group8_steps(F&& f) {
  f(std::integral_constant<int, 0>{});
  f(std::integral_constant<int, 1>{});
  f(std::integral_constant<int, 2>{});
}

// Workgroup barrier for data exchanged through LDS: waits for this wavefront's LDS operations only.  (__syncthreads
// also waits for every global load and store in flight: for the results just stored, a microsecond at the end of a
// kernel that lasts ten, and for refill loads that nobody will use.)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

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

// One wavefront ranks one token from its float64 logits z[0..E): softmax in float32 (row maximum subtracted),
// k rounds of arg-max on the float64 logits (ties -> lower expert index), weights p or p / sum of the selected.
// Returns the j-th selected expert in lane j < k (0 in the other lanes).
__device__ __forceinline__ int rank_token(const double* z, int lane, int E, int k, int renorm, int t,
                                          int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                          float* __restrict__ probs) {
  // each lane owns experts lane, lane+64, ...
  double zd[4];
  float zf[4];
  float mx = -INFINITY;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int e = lane + 64 * s;
    zd[s] = e < E ? z[e] : -INFINITY;
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
  return isel;
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
    rank_token(zs + q * Epad, lane, E, k, renorm, t, topk_idx, topk_w, probs);
  }
}

// Few tokens (T <= FEW_MAX_T; E = 4, 8, 16, 32 or 64): one workgroup per token, so that the whole router matrix
// is not read through one compute unit's handful of wavefronts, with loads that are contiguous across the
// wavefront: a router row is E/4 chunks of four floats; lane (r, c) of a wavefront reads chunk c of the r-th of
// the 64 / (E/4) rows that one wave-wide load covers, and accumulates those four logits in float64 (exact
// products, see above) over its share of the rows.  The sums meet across the row groups of a wavefront by a
// butterfly, across the wavefronts in wavefront order, and wavefront 0 ranks the token.
constexpr int FEW_MAX_T = 16;
constexpr int FEW_WAVES = 16;  // (all the loads of a token are in flight in two batches at d_model = 2048)
constexpr int FEW_THREADS = FEW_WAVES * 64;

template <typename XT>
__global__ __launch_bounds__(FEW_THREADS) void gate_few_kernel(
    const XT* __restrict__ x, const float* __restrict__ wr, const float* __restrict__ br, int T, int d, int E, int k,
    int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w, float* __restrict__ probs,
    int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ a2r, int32_t* __restrict__ r2a,
    int32_t* __restrict__ clear8) {
  __shared__ double part[FEW_WAVES][64];
  __shared__ double zrow[64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x;
  const int cpr = E >> 2, rpi = 64 / cpr;  // chunks per row, rows per wave-wide load
  const int r = lane / cpr, c = lane % cpr;
  const XT* xt = x + (size_t)t * d;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll 16
  for (int row = wave * rpi + r; row < d; row += FEW_WAVES * rpi) {
    const float4 w4 = *reinterpret_cast<const float4*>(wr + (size_t)row * E + 4 * c);
    float xv;
    if constexpr (sizeof(XT) == 2) xv = bf16_to_f32(xt[row]);
    else xv = xt[row];
    const double xd = (double)xv;
    a0 = fma(xd, (double)w4.x, a0);
    a1 = fma(xd, (double)w4.y, a1);
    a2 = fma(xd, (double)w4.z, a2);
    a3 = fma(xd, (double)w4.w, a3);
  }
  for (int m = cpr; m < 64; m <<= 1) {  // lanes with the same chunk sit cpr apart
    a0 += shfl_xor_f64(a0, m);
    a1 += shfl_xor_f64(a1, m);
    a2 += shfl_xor_f64(a2, m);
    a3 += shfl_xor_f64(a3, m);
  }
  if (lane < cpr) {
    part[wave][4 * c] = a0; part[wave][4 * c + 1] = a1; part[wave][4 * c + 2] = a2; part[wave][4 * c + 3] = a3;
  }
  __syncthreads();
  if ((int)threadIdx.x < E) {
    double zsum = 0.0;
#pragma unroll
    for (int w = 0; w < FEW_WAVES; ++w) zsum += part[w][threadIdx.x];
    zrow[threadIdx.x] = zsum + (br ? (double)br[threadIdx.x] : 0.0);
  }
  __syncthreads();
  if (wave != 0) return;
  const int sel = rank_token(zrow, lane, E, k, renorm, t, topk_idx, topk_w, probs);
  // A step of ONE token (counts != NULL; T == 1): its dispatch tables follow from the selection at once.  The k
  // experts are distinct and get one row each (the capacity is at least one, so nothing is dropped); rows are
  // ordered by expert; assignment j (= j*T + t with T = 1) is the j-th choice.
  if (counts) {
    unsigned long long chosen = 0;  // bit e: expert e selected (E <= 64)
    for (int j = 0; j < k; ++j) chosen |= 1ull << __shfl(sel, j, 64);
    if (lane < E) {
      counts[lane] = (int)((chosen >> lane) & 1ull);
      offsets[lane] = __popcll(chosen & ((1ull << lane) - 1ull));
    }
    if (lane == 0) offsets[E] = k;
    if (lane < k) {
      const int row = __popcll(chosen & ((1ull << sel) - 1ull));
      a2r[lane] = row;
      r2a[row] = lane;
    }
    if (clear8 && lane < 8) clear8[lane] = 0;
  }
}

// the shapes the kernel above is written for
bool gate_few_applies(const moe_config* cfg, const float* w_router) {
  const int E = cfg->E;
  return tuning(MOE_TUNE_FEW_TOKEN_KERNELS) != 0 && cfg->T <= FEW_MAX_T && (E == 4 || E == 8 || E == 16 || E == 32 || E == 64) &&
         (reinterpret_cast<uintptr_t>(w_router) & 15) == 0;
}

template <typename XT>
int32_t launch_few(const moe_config* cfg, const void* x, const float* w_router, const float* b_router, int32_t* topk_idx,
                   float* topk_w, float* probs, hipStream_t s, int32_t* counts = nullptr, int32_t* offsets = nullptr,
                   int32_t* a2r = nullptr, int32_t* r2a = nullptr, int32_t* clear8 = nullptr) {
  hipLaunchKernelGGL(gate_few_kernel<XT>, dim3(cfg->T), dim3(FEW_THREADS), 0, s, (const XT*)x, w_router, b_router, cfg->T,
                     cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w, probs, counts, offsets, a2r, r2a, clear8);
  return check_hip(hipGetLastError(), "gate launch");
}

// ------------------------------------------------------------------------------------------------
// Fast path.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int FT_TOK = 16;           // tokens per workgroup (one 16-token MFMA tile)
constexpr int FT_KC = 64;            // K chunk: two 16x16x32 MFMA steps
constexpr int FT_ROW = (FT_KC + 8) * 2;  // LDS row of one expert's chunk, padded to 144 B (conflict-free reads)
// neighbours among the k+1 leading logits closer than this times the token's largest |logit| -> exact recompute
// (the accumulation error scales with the data; for inputs of unit variance this is about 1e-4)
constexpr float GATE_MARGIN_REL = 1.0f / 32768.0f;

__device__ __forceinline__ uint32_t bf16_bits_rne(float f) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f); }

// Softmax (fp32) + top-k of one token by a group of 8 adjacent lanes.  Lane `sub` of the group holds the
// float64 logits of experts sub, sub+8, ... (NPL of them, -inf beyond E).  k+1 rounds of group-wide
// arg-max (ties -> lower expert) pick the experts in rank order; the extra round only measures the gap
// to the first expert NOT selected.  Returns true (to every lane of the group) if two neighbours among
// those k+1 logits are closer than `margin`.
template <int NPL>
__device__ __forceinline__ bool finalize_group(double (&z)[NPL], int sub, int E, int k, int renorm, float margin,
                                               int32_t* __restrict__ idx_out, float* __restrict__ w_out,
                                               float* __restrict__ probs_out, bool mark_close = false) {
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NPL; ++i) mx = fmaxf(mx, (float)z[i]);
  group8_steps([&](auto st) { mx = fmaxf(mx, group8_partner<decltype(st)::value>(mx)); });
  float ex[NPL], sum = 0.f;
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    ex[i] = (sub + 8 * i) < E ? expf((float)z[i] - mx) : 0.f;
    sum += ex[i];
  }
  // (the same pairs in the same order in every lane of the group: all eight hold the same sum, bit for bit)
  group8_steps([&](auto st) { sum += group8_partner<decltype(st)::value>(sum); });
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    ex[i] = ex[i] / sum;
    if (probs_out && (sub + 8 * i) < E) probs_out[sub + 8 * i] = ex[i];
  }
  float my_w = 0.f, wsum = 0.f;
  int my_idx = 0;
  double prev = INFINITY;
  bool close = false;
  for (int r = 0; r <= k; ++r) {
    double bz = -INFINITY;
    int be = 0x7fffffff;
    float bp = 0.f;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int e = sub + 8 * i;
      if (e < E && (z[i] > bz || (z[i] == bz && e < be))) { bz = z[i]; be = e; bp = ex[i]; }
    }
    group8_steps([&](auto st) {
      constexpr int S = decltype(st)::value;
      const double oz = group8_partner<S>(bz);
      const int oe = group8_partner<S>(be);
      const float op = group8_partner<S>(bp);
      if (oz > bz || (oz == bz && oe < be)) { bz = oz; be = oe; bp = op; }
    });
#pragma unroll
    for (int i = 0; i < NPL; ++i)
      if (sub + 8 * i == be) z[i] = -INFINITY;  // retire the winner (every lane of the group agrees on be)
    if (r < k) {
      if (sub == r) { my_idx = be; my_w = bp; }
      wsum += bp;
    }
    if (r > 0) close |= (float)(prev - bz) < margin;
    prev = bz;
  }
  if (sub < k) {
    idx_out[sub] = my_idx;
    float w = renorm ? my_w / wsum : my_w;
    // mark_close: a token within the margin carries the sign bit on its first weight (a probability, never
    // negative otherwise) until the kernel that recomputes such tokens has replaced its results
    if (mark_close && close && sub == 0) w = __uint_as_float(__float_as_uint(w) | 0x80000000u);
    w_out[sub] = w;
  }
  return close;
}

// EB = number of 16-expert blocks (E <= 16*EB).  One workgroup = 16 tokens (one MFMA token tile); its NWV
// wavefronts split the K range chunk by chunk and meet once, to add their partial logits.  A wavefront
// works through a chunk one expert block at a time, re-using one staging area of 16 experts (its LDS
// operations execute in order), so that eight wavefronts fit where the router is wide: with 64 experts a
// wavefront's chain of split, stage and multiply is four times as long as with 16, and the kernel's time
// is the length of that chain.  VEC: the router weights can be read four experts at a time (E a multiple
// of 4, 16-byte aligned base).
template <int EB>
constexpr int gate_waves() { return EB == 1 ? 4 : 8; }

// TT = 16-token tiles per workgroup.  The split of the router into its three pieces is the larger part of a
// workgroup's work and does not depend on the tokens: two tiles share it (and the 64 KB of router a workgroup reads
// per 16 experts), which is worth it once there are enough tokens to keep every CU busy with half as many workgroups.
template <int EB, bool VEC, int TT>
__global__ __launch_bounds__(gate_waves<EB>() * 64) void gate_mfma_kernel(const uint16_t* __restrict__ x, const float* __restrict__ wr,
                                                        const float* __restrict__ br, int T, int d, int E, int k,
                                                        int renorm, int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w, float* __restrict__ probs) {
  constexpr int EP = EB * 16;
  constexpr int NPL = EP / 8;                    // logits per lane in the 8-lane finalisation groups
  constexpr int NWV = gate_waves<EB>();
  constexpr int W_WAVE_BYTES = 3 * 16 * FT_ROW;  // one wavefront's hi/mid/lo pieces of one expert block's chunk
  constexpr int PF = EB == 1 ? 4 : 2;            // chunks in flight per wavefront (register-staged)
  constexpr int NTOK = FT_TOK * TT;              // tokens per workgroup
  static_assert(NTOK <= 32 && NTOK * 8 <= NWV * 64, "one flag bit and eight finalising lanes per token");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_flag[NTOK];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* wl = smem + wave * W_WAVE_BYTES;
  const int t0 = blockIdx.x * NTOK;
  const int tl = lane & 15, kq = lane >> 4;  // MFMA operand coordinates of this lane

  // activation rows of this lane, one per token tile (clamped: tail tokens recompute the last row, never stored)
  const uint16_t* xrow[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) xrow[tt] = x + (size_t)min(t0 + tt * FT_TOK + tl, T - 1) * d + kq * 16;

  double zacc[TT][EB][4];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int b = 0; b < EB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) zacc[tt][b][r] = 0.0;

  // router-weight micro-tiles of this lane: 4 consecutive k x 4 consecutive experts each
  // (micro-tile m of a lane belongs to expert block m: expert group m*4 + lane%4, K group lane/4)
  constexpr int MT_PER_LANE = (FT_KC / 4) * (EP / 4) / 64;  // = EB
  const int n_chunks = d / FT_KC;

  // PF register stages.  Every stage load is unconditional (a chunk index past the end re-reads the last
  // chunk and is never used), so the number of loads in flight is fixed and the wait before a stage's
  // first use can leave the younger stages outstanding.
  u32x4 xa[PF][TT][2];
  float wv[PF][MT_PER_LANE][4][4];
#define GATE_LOAD_STAGE(s_, c_)                                                                         \
  {                                                                                                     \
    const int k0_ = min((c_), n_chunks - 1) * FT_KC;                                                    \
    _Pragma("unroll") for (int tt_ = 0; tt_ < TT; ++tt_) {                                              \
      xa[s_][tt_][0] = *reinterpret_cast<const u32x4*>(xrow[tt_] + k0_);                                \
      xa[s_][tt_][1] = *reinterpret_cast<const u32x4*>(xrow[tt_] + k0_ + 8);                            \
    }                                                                                                   \
    _Pragma("unroll") for (int m = 0; m < MT_PER_LANE; ++m) {                                           \
      const int eg = m * 4 + (lane & 3), kg = lane >> 2;                                                \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                   \
        const float* wp = wr + (size_t)(k0_ + kg * 4 + i) * E;                                          \
        if (VEC) {                                                                                      \
          const f32x4 v = *reinterpret_cast<const f32x4*>(wp + min(eg * 4, E - 4));                     \
          const bool ok = eg * 4 < E;                                                                   \
          wv[s_][m][i][0] = ok ? v[0] : 0.f; wv[s_][m][i][1] = ok ? v[1] : 0.f;                         \
          wv[s_][m][i][2] = ok ? v[2] : 0.f; wv[s_][m][i][3] = ok ? v[3] : 0.f;                         \
        } else {                                                                                        \
          _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                               \
            const int e = eg * 4 + j;                                                                   \
            const float v = wp[min(e, E - 1)];                                                          \
            wv[s_][m][i][j] = e < E ? v : 0.f;                                                          \
          }                                                                                             \
        }                                                                                               \
      }                                                                                                 \
    }                                                                                                   \
  }

  // chunks wave, wave+NWV, ...  The LDS staging area is private to the wavefront and LDS operations of one
  // wavefront execute in order, so no barrier is needed inside this loop.
#pragma unroll
  for (int s = 0; s < PF; ++s) GATE_LOAD_STAGE(s, wave + NWV * s)
  for (int base = wave; base < n_chunks; base += NWV * PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      const int c = base + NWV * s;
      const bool live = c < n_chunks;  // uniform
      bf16x8 xb[TT][2];
      f32x4 acc[TT][EB];
      if (live) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          xb[tt][0] = __builtin_bit_cast(bf16x8, xa[s][tt][0]);
          xb[tt][1] = __builtin_bit_cast(bf16x8, xa[s][tt][1]);
        }
        // one expert block at a time: split its router weights into three bf16 pieces, stage them
        // K-contiguous per expert, multiply
#pragma unroll
        for (int m = 0; m < MT_PER_LANE; ++m) {
          const int egl = lane & 3, kg = lane >> 2;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint32_t hi[4], mid[4], lo[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float w = wv[s][m][i][j];
              hi[i] = bf16_bits_rne(w);
              const float r1 = w - __uint_as_float(hi[i] << 16);
              mid[i] = bf16_bits_rne(r1);
              const float r2 = r1 - __uint_as_float(mid[i] << 16);
              lo[i] = bf16_bits_rne(r2);
            }
            unsigned char* row = wl + (egl * 4 + j) * FT_ROW + kg * 8;
            u32x2 v;
            v.x = hi[0] | (hi[1] << 16); v.y = hi[2] | (hi[3] << 16);
            *reinterpret_cast<u32x2*>(row) = v;
            v.x = mid[0] | (mid[1] << 16); v.y = mid[2] | (mid[3] << 16);
            *reinterpret_cast<u32x2*>(row + 16 * FT_ROW) = v;
            v.x = lo[0] | (lo[1] << 16); v.y = lo[2] | (lo[3] << 16);
            *reinterpret_cast<u32x2*>(row + 2 * 16 * FT_ROW) = v;
          }
          asm volatile("" ::: "memory");  // keep the LDS reads below the LDS writes above (same wavefront: in order)
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) acc[tt][m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int p = 0; p < 3; ++p) {
              const bf16x8 wf = *reinterpret_cast<const bf16x8*>(wl + (p * 16 + tl) * FT_ROW + kq * 32 + s2 * 16);
#pragma unroll
              for (int tt = 0; tt < TT; ++tt)
                acc[tt][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xb[tt][s2], acc[tt][m], 0, 0, 0);
            }
          asm volatile("" ::: "memory");  // ... and the next block's writes below these reads
        }
      }
      GATE_LOAD_STAGE(s, c + NWV * PF)  // refill this register stage
      if (live) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
          for (int b = 0; b < EB; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) zacc[tt][b][r] += (double)acc[tt][b][r];
      }
    }
  }
#undef GATE_LOAD_STAGE
  lds_barrier();     // every wavefront is done with its staging area

  // ---- cross-wavefront sum of the partial logits (float64) and per-token finalisation ------------
  double* part = reinterpret_cast<double*>(smem);  // [NWV][EP][NTOK]
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int b = 0; b < EB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        part[((size_t)wave * EP + b * 16 + kq * 4 + r) * NTOK + tt * FT_TOK + tl] = zacc[tt][b][r];
  lds_barrier();
  if (tid < NTOK * 8) {
    const int tok = tid >> 3, sub = tid & 7;
    const int t = t0 + tok;
    double z[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      const int e = sub + 8 * i;
      double v = -INFINITY;
      if (e < E) {
        v = part[(size_t)e * NTOK + tok];
#pragma unroll
        for (int w = 1; w < NWV; ++w) v += part[((size_t)w * EP + e) * NTOK + tok];
        if (br) v += (double)br[e];
      }
      z[i] = v;
    }
    const int tc = min(t, T - 1);  // tail tokens run the same code on the last row, without storing
    float zmax = 0.f;
#pragma unroll
    for (int i = 0; i < NPL; ++i)
      if (sub + 8 * i < E) zmax = fmaxf(zmax, fabsf((float)z[i]));
    group8_steps([&](auto st) { zmax = fmaxf(zmax, group8_partner<decltype(st)::value>(zmax)); });
    bool flag = false;
    if (t < T)
      flag = finalize_group<NPL>(z, sub, E, k, renorm, GATE_MARGIN_REL * zmax, topk_idx + (size_t)tc * k, topk_w + (size_t)tc * k,
                                 probs ? probs + (size_t)tc * E : nullptr);
    if (sub == 0) s_flag[tok] = flag ? 1 : 0;
  }
  lds_barrier();

  // ---- exact recompute of the rare tokens whose ranking is within the margin -------------------
  // Each wavefront takes a contiguous K range; a load instruction covers whole router rows (lane = expert
  // quad + row slot), so that it is coalesced and many of them can be in flight: a token flagged in one
  // workgroup delays the whole kernel by the time this takes.  The products are exact in float64 and so is
  // their sum up to rounding at 2^-53, far below any gap that can decide a ranking.  The flags are turned
  // into one wave-uniform mask first (no LDS read per token).
  uint32_t flagged = (uint32_t)__ballot(lane < NTOK && s_flag[lane & (NTOK - 1)] != 0);
  flagged = __builtin_amdgcn_readfirstlane(flagged);
  constexpr int QN = EP / 4;    // expert quads per router row
  constexpr int RPI = 64 / QN;  // router rows per load instruction of a wavefront
  double* zpart = part;         // [NWV][EP]
  double* zex = part + NWV * EP;  // [EP]
  const int q = lane % QN, rs = lane / QN;
  const int rows_per_wave = d / NWV;  // d is a multiple of 64: a whole number of load instructions
  const bool qlive = q * 4 < E;
  while (flagged) {
    const int tt = __builtin_ctz(flagged);
    flagged &= flagged - 1;
    const int t = t0 + tt;
    const uint16_t* xt = x + (size_t)t * d;
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    const int r_end = (wave + 1) * rows_per_wave;
#pragma unroll 8
    for (int r = wave * rows_per_wave + rs; r < r_end; r += RPI) {
      const double xv = (double)bf16_to_f32(xt[r]);
      const float* wp = wr + (size_t)r * E + q * 4;
      float w[4] = {0.f, 0.f, 0.f, 0.f};
      if (VEC) {
        if (qlive) {  // E is a multiple of 4: q*4 + 3 < E
          const f32x4 v = *reinterpret_cast<const f32x4*>(wp);
          w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (q * 4 + j < E) w[j] = wp[j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) a[j] = fma(xv, (double)w[j], a[j]);
    }
#pragma unroll
    for (int m = QN; m < 64; m <<= 1)
#pragma unroll
      for (int j = 0; j < 4; ++j) a[j] += shfl_xor_f64(a[j], m);
    if (rs == 0) {
#pragma unroll
      for (int j = 0; j < 4; ++j) zpart[wave * EP + q * 4 + j] = a[j];
    }
    lds_barrier();
    if (tid < E) {
      double v = zpart[tid];
#pragma unroll
      for (int w = 1; w < NWV; ++w) v += zpart[w * EP + tid];
      zex[tid] = v + (br ? (double)br[tid] : 0.0);
    }
    lds_barrier();
    if (tid < 8) {
      double z[NPL];
#pragma unroll
      for (int i = 0; i < NPL; ++i) z[i] = (tid + 8 * i) < E ? zex[tid + 8 * i] : -INFINITY;
      finalize_group<NPL>(z, tid, E, k, renorm, 0.f, topk_idx + (size_t)t * k, topk_w + (size_t)t * k,
                          probs ? probs + (size_t)t * E : nullptr);
    }
    lds_barrier();
  }
}

template <int EB>
int32_t launch_fast(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                    int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s) {
  constexpr int EP = EB * 16;
  constexpr int NWV = gate_waves<EB>();
  const size_t w_bytes = (size_t)NWV * 3 * 16 * FT_ROW;
  // two token tiles per workgroup for narrow routers once that still leaves a workgroup for every CU
  constexpr int TT_MAX = EB == 1 ? 2 : 1;
  const int tt = (TT_MAX == 2 && cfg->T >= 2 * FT_TOK * 256) ? 2 : 1;  // (256 CUs)
  const size_t z_bytes = (size_t)NWV * EP * FT_TOK * tt * sizeof(double) + 256;
  const size_t shmem = w_bytes > z_bytes ? w_bytes : z_bytes;
  const bool vec = cfg->E % 4 == 0 && ((uintptr_t)w_router & 15) == 0;
  auto kern = tt == 2 ? (vec ? gate_mfma_kernel<EB, true, TT_MAX> : gate_mfma_kernel<EB, false, TT_MAX>)
                      : (vec ? gate_mfma_kernel<EB, true, 1> : gate_mfma_kernel<EB, false, 1>);
  if (shmem > 65536) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(gate LDS)");
  }
  hipLaunchKernelGGL(kern, dim3((cfg->T + FT_TOK * tt - 1) / (FT_TOK * tt)), dim3(NWV * 64), shmem, s, (const uint16_t*)x, w_router,
                     b_router, cfg->T, cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w, probs);
  return check_hip(hipGetLastError(), "gate launch");
}


// ------------------------------------------------------------------------------------------------
// Fast path on a pre-split router (moe_pack_router): the HBM-rate gate.
//
// The split of the float32 router into three bfloat16 pieces does not depend on the tokens, so it is done once,
// outside the hot path, into the order the MFMA reads its operand in: rows of the packed matrix are
// (piece, expert) pairs, row = piece * E + expert, padded with zero rows to FR blocks of 32; the contraction
// index runs in stages of KC = 16 G values, and inside a stage the lower 32 lanes of a wavefront hold its
// first KC/2 values and the upper 32 lanes the others (a dot product does not care about the order, as long as
// both operands use the same one): that way a lane's share of a token row is one contiguous run of KC bytes and
// a wavefront's loads of one stage cover whole cache lines of every token row.  A fragment (stage, sub-step,
// row block) is 1 KB, contiguous, in that order.
//
// One workgroup = NT = 32 NB tokens, eight wavefronts that split the contraction index in runs of a few stages.  A wavefront multiplies v_mfma_f32_32x32x16_bf16 tiles, router rows x tokens, and
// every product is exact in float32 (a bfloat16 piece times a bfloat16 activation), so the only rounding is the
// float32 accumulation over the wavefront's share of the contraction index; the eight partial sums and the three
// pieces of an expert meet in float64 through LDS.  No staging through LDS on the way in, no conversion in the
// loop: the loop is loads and MFMAs, and the kernel runs at the rate the token rows arrive from HBM.
//
// Ranking must equal the ranking of the exactly computed logits.  The partial sums carry errors of about
// 2^-24 times their own magnitude, so a token is marked when two neighbours among its k+1 leading logits are
// closer than 2^-15 times the largest sum over the wavefronts of |partial logit| of that token (a margin that
// scales with the data; about 1e-4 for inputs of unit variance): the mark is the sign bit of its first gate
// weight, and gate_fix_kernel, launched behind this kernel, recomputes the marked tokens with float64
// accumulation of the exact products, from the float32 router itself.
#ifndef GATE_REL_MARGIN_VALUE
#define GATE_REL_MARGIN_VALUE (1.0f / 32768.0f)
#endif
constexpr float GATE_REL_MARGIN = GATE_REL_MARGIN_VALUE;
constexpr int GP_WAVES = 8;

__host__ __device__ constexpr int gate_frags(int E) { return (3 * E + 31) / 32; }        // row blocks of the packed router
__host__ __device__ constexpr int gate_substeps(int FR) { return FR <= 3 ? 4 : 2; }      // MFMA sub-steps per stage

// one thread per 16-byte piece of the packed router
__global__ __launch_bounds__(256) void pack_router_kernel(const float* __restrict__ wr, uint16_t* __restrict__ dst, int d, int E,
                                                          int FR, int G) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)(d / (16 * G)) * G * FR * 64;
  if (i >= total) return;
  const int lane = (int)(i % 64);
  const size_t frag = i / 64;
  const int fr = (int)(frag % FR), s = (int)((frag / FR) % G);
  const size_t c = frag / ((size_t)FR * G);
  const int row = 32 * fr + (lane & 31), h = lane >> 5;
  const int piece = row / E, e = row - piece * E;
  const size_t k0 = c * (16 * G) + (size_t)(8 * G) * h + 8 * s;
  uint32_t out[4] = {0u, 0u, 0u, 0u};
  if (piece < 3) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float w = wr[(k0 + j) * E + e];
      const uint32_t hi = bf16_bits_rne(w);
      const float r1 = w - __uint_as_float(hi << 16);      // exact: the leading 8 bits of the significand are gone
      const uint32_t mid = bf16_bits_rne(r1);
      const float r2 = r1 - __uint_as_float(mid << 16);    // exact; at most 8 significant bits are left
      const uint32_t lo = bf16_bits_rne(r2);
      const uint32_t v = piece == 0 ? hi : piece == 1 ? mid : lo;
      out[j >> 1] |= v << (16 * (j & 1));
    }
  }
  *reinterpret_cast<u32x4*>(dst + i * 8) = u32x4{out[0], out[1], out[2], out[3]};
}

typedef float f32x16 __attribute__((ext_vector_type(16)));

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N - 1>{}), unrolled
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

// One token's logits with float64 accumulation of the exact products of the float32 router and the activations,
// then softmax and ranking on those values: the whole workgroup of GP_WAVES wavefronts works on the token.  Every
// wavefront takes a contiguous range of router rows; a load instruction covers whole rows (lane = expert quad + row
// slot) and sixteen of them are in flight.  lds: (GP_WAVES + 1) * 64 doubles; the caller synchronises before.
__device__ __forceinline__ void exact_token(const uint16_t* __restrict__ x, const float* __restrict__ wr, const float* __restrict__ br,
                                            int t, int d, int E, int k, int renorm, int32_t* __restrict__ topk_idx,
                                            float* __restrict__ topk_w, float* __restrict__ probs, double* lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // expert quads per router row (a power of two that covers E) and router rows per wave-wide load instruction
  const int QN = E <= 4 ? 1 : E <= 8 ? 2 : E <= 16 ? 4 : E <= 32 ? 8 : 16, RPI = 64 / QN;
  double* zpart = lds;                  // [GP_WAVES][64]
  double* zex = lds + GP_WAVES * 64;    // [64]
  const int q = lane % QN, rs = lane / QN;
  const int rows_per_wave = d / GP_WAVES;   // d is a multiple of 64
  const bool vec = (E & 3) == 0 && (reinterpret_cast<uintptr_t>(wr) & 15) == 0;
  const uint16_t* xt = x + (size_t)t * d;
  double a[4] = {0.0, 0.0, 0.0, 0.0};
  // All loads of a batch are issued before the first is used, and the trip count is the same for every lane (rows
  // past the wavefront's range re-read its first row and are multiplied by zero): a loop that can leave early
  // makes the compiler wait for every load where it stands, and the token then costs one memory latency per
  // router row instead of one per batch.
  const int r_begin = wave * rows_per_wave, r_end = r_begin + rows_per_wave;
  const int n_it = (rows_per_wave + RPI - 1) / RPI;
  const bool q_live = q * 4 < E;
  const int last = q_live ? min(3, E - 1 - q * 4) : 0;   // scalar loads of a ragged last quad stay inside the row
  auto rows = [&](auto is_vec, auto batch) {
    constexpr int BATCH = decltype(batch)::value;
    for (int it0 = 0; it0 < n_it; it0 += BATCH) {
      float w4[BATCH][4];
      uint16_t xb[BATCH];
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int r = r_begin + rs + (it0 + j) * RPI;
        const int rc = r < r_end ? r : r_begin;
        const float* wq = q_live ? wr + (size_t)rc * E + q * 4 : wr;   // quads past the last expert read the first row
        if constexpr (decltype(is_vec)::value) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(wq);
          w4[j][0] = v[0]; w4[j][1] = v[1]; w4[j][2] = v[2]; w4[j][3] = v[3];
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c) w4[j][c] = wq[min(c, last)];
        }
        xb[j] = xt[rc];
      }
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int r = r_begin + rs + (it0 + j) * RPI;
        const double xd = r < r_end ? (double)bf16_to_f32(xb[j]) : 0.0;
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = fma(xd, (q * 4 + c < E) ? (double)w4[j][c] : 0.0, a[c]);
      }
    }
  };
  if (vec) rows(std::true_type{}, std::integral_constant<int, 16>{});
  else rows(std::false_type{}, std::integral_constant<int, 16>{});
  for (int m = QN; m < 64; m <<= 1)
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] += shfl_xor_f64(a[j], m);
  if (rs == 0) {
#pragma unroll
    for (int j = 0; j < 4; ++j) zpart[wave * 64 + q * 4 + j] = a[j];
  }
  __syncthreads();
  if (tid < E) {
    double v = zpart[tid];
#pragma unroll
    for (int w = 1; w < GP_WAVES; ++w) v += zpart[w * 64 + tid];
    zex[tid] = v + (br ? (double)br[tid] : 0.0);
  }
  __syncthreads();
  if (tid < 8) {
    double z[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (tid + 8 * i) < E ? zex[tid + 8 * i] : -INFINITY;
    finalize_group<8>(z, tid, E, k, renorm, 0.f, topk_idx + (size_t)t * k, topk_w + (size_t)t * k,
                      probs ? probs + (size_t)t * E : nullptr);
  }
}

// Recomputes the tokens that gate_packed_kernel marked (sign bit of the first gate weight): one workgroup looks at
// FIX_TOKENS tokens and works through the marked ones (almost always none, rarely one), replacing indices, weights
// and probabilities.  Launched behind every gate_packed_kernel: inside that kernel a marked token would hold up its
// whole workgroup, and with it the kernel, for the time of a chain of dependent loads.
constexpr int FIX_TOKENS = 64;
__global__ __launch_bounds__(GP_WAVES * 64) void gate_fix_kernel(const uint16_t* __restrict__ x, const float* __restrict__ wr,
                                                                 const float* __restrict__ br, int T, int d, int E, int k, int renorm,
                                                                 int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                                 float* __restrict__ probs) {
  __shared__ double lds[(GP_WAVES + 1) * 64];
  const int lane = threadIdx.x & 63;
  const int t0 = blockIdx.x * FIX_TOKENS;
  static_assert(FIX_TOKENS == 64, "one ballot");
  const int t = t0 + lane;
  unsigned long long todo = __ballot(t < T && (__float_as_uint(topk_w[(size_t)min(t, T - 1) * k]) >> 31) != 0);
  while (todo) {
    const int st = __builtin_ctzll(todo);
    todo &= todo - 1;
    __syncthreads();
    exact_token(x, wr, br, t0 + st, d, E, k, renorm, topk_idx, topk_w, probs, lds);
  }
}

// What follows the contraction in the gate kernels on a packed router: acc[nb][fr] holds this wavefront's partial
// sums (router rows x tokens, the MFMA's accumulator layout) for the NT = 32 NB tokens from t0 on.  The partial sums
// of the eight wavefronts and the three pieces of every expert meet in float64 through LDS (smem: room for the
// partial-sum matrices), then softmax, ranking and the margin test per token; tokens within the margin are
// marked for gate_fix_kernel.
template <int FR, int NB>
__device__ __forceinline__ void gate_finish(f32x16 (&acc)[NB][FR], unsigned char* smem, int t0, const float* __restrict__ br, int T,
                                            int E, int k, int renorm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                            float* __restrict__ probs) {
  constexpr int NT = 32 * NB, RW = 32 * FR;
  constexpr int STRIDE = NT + 8;  // floats between the rows of a partial-sum matrix (conflict-free reads and writes)
  constexpr int NPL = (32 * FR / 3 + 7) / 8;  // logits per lane of an 8-lane group (covers every E of this FR)
  // all eight partial-sum matrices in LDS at once, or four and two rounds
  constexpr bool TWO_ROUNDS = (size_t)GP_WAVES * RW * STRIDE * 4 > 150 * 1024;
  constexpr int SLOTS = TWO_ROUNDS ? GP_WAVES / 2 : GP_WAVES;
  float* part = reinterpret_cast<float*>(smem);  // [SLOTS][RW][STRIDE]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tok = lane & 31, h = lane >> 5;
  // ---- the partial sums meet in LDS: part[slot][row][token] -------------------------------------
  auto put = [&](int slot) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int fr = 0; fr < FR; ++fr)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 32 * fr + 8 * (v >> 2) + 4 * h + (v & 3);
          part[((size_t)slot * RW + row) * STRIDE + 32 * nb + tok] = acc[nb][fr][v];
        }
  };
  if constexpr (TWO_ROUNDS) {
    // the upper four wavefronts hand their sums to the lower four (one float32 addition: 2^-24 of a partial sum)
    if (wave >= SLOTS) put(wave - SLOTS);
    __syncthreads();
    if (wave < SLOTS) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = 32 * fr + 8 * (v >> 2) + 4 * h + (v & 3);
            acc[nb][fr][v] += part[((size_t)wave * RW + row) * STRIDE + 32 * nb + tok];
          }
    }
    __syncthreads();
    if (wave < SLOTS) put(wave);
  } else {
    put(wave);
  }
  __syncthreads();

  // ---- per token: float64 sum over wavefronts and pieces, float32 softmax, ranking, margin test ----------
  for (int base = 0; base < NT; base += GP_WAVES * 8) {
    const int slot_tok = base + (tid >> 3), sub = tid & 7;
    const int t = t0 + slot_tok;
    if (slot_tok < NT) {   // (uniform per 8-lane group)
      double z[NPL];
      float zabs = 0.f;
#pragma unroll
      for (int i = 0; i < NPL; ++i) {
        const int e = sub + 8 * i;
        double v = -INFINITY;
        if (e < E) {
          v = 0.0;
          float a = 0.f;
          for (int w = 0; w < SLOTS; ++w) {
            const float* pw = part + ((size_t)w * RW + e) * STRIDE + slot_tok;
            const double pz = (double)pw[0] + (double)pw[(size_t)E * STRIDE] + (double)pw[(size_t)2 * E * STRIDE];
            v += pz;
            a += fabsf((float)pz);
          }
          zabs = fmaxf(zabs, a);
          if (br) v += (double)br[e];
        }
        z[i] = v;
      }
      group8_steps([&](auto st) { zabs = fmaxf(zabs, group8_partner<decltype(st)::value>(zabs)); });
      const int tc = min(t, T - 1);
      if (t < T)
        finalize_group<NPL>(z, sub, E, k, renorm, GATE_REL_MARGIN * zabs, topk_idx + (size_t)tc * k, topk_w + (size_t)tc * k,
                            probs ? probs + (size_t)tc * E : nullptr, true);
    }
  }

}

template <int FR, int NB>
__global__ __launch_bounds__(GP_WAVES * 64) void gate_packed_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wp,
                                                                    const float* __restrict__ wr, const float* __restrict__ br, int T,
                                                                    int d, int E, int k, int renorm, int32_t* __restrict__ topk_idx,
                                                                    float* __restrict__ topk_w, float* __restrict__ probs) {
  constexpr int G = gate_substeps(FR), KC = 16 * G, NT = 32 * NB;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tok = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * NT;
  const int n_stages = d / KC;

  // this lane's run of every token row (tail tokens recompute the last row and are never stored)
  const uint16_t* xrow[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) xrow[nb] = x + (size_t)min(t0 + 32 * nb + tok, T - 1) * d + (KC / 2) * h;
  const uint16_t* wlane = wp + lane * 8;

  f32x16 acc[NB][FR];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int fr = 0; fr < FR; ++fr)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[nb][fr][v] = 0.f;

  // PF register stages in flight.  Every stage load is unconditional (a stage index past the end re-reads the
  // last stage) and every stage is multiplied, with the token fragments of a stage past the end replaced by
  // zeros (which add nothing): loads and uses then sit in straight-line code, the compiler can neither sink a
  // load into a branch next to its use nor merge the stages' registers, and a scheduling barrier after each
  // group of loads keeps them ahead of the multiplications of the older stages.
  constexpr int STAGE_REGS = (NB + FR) * G * 4;
  constexpr int PF = STAGE_REGS <= 32 ? 4 : STAGE_REGS <= 48 ? 3 : 2;
  u32x4 xs[PF][NB][G], ws[PF][G][FR];
  auto load_stage = [&](auto b_tag, int c) {
    constexpr int b = decltype(b_tag)::value;
    const int cc = min(c, n_stages - 1);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int s = 0; s < G; ++s) xs[b][nb][s] = *reinterpret_cast<const u32x4*>(xrow[nb] + (size_t)cc * KC + 8 * s);
#pragma unroll
    for (int s = 0; s < G; ++s)
#pragma unroll
      for (int fr = 0; fr < FR; ++fr)
        ws[b][s][fr] = *reinterpret_cast<const u32x4*>(wlane + (((size_t)cc * G + s) * FR + fr) * 512);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto multiply = [&](auto b_tag, int c) {
    constexpr int b = decltype(b_tag)::value;
    const uint32_t keep = c < n_stages ? 0xffffffffu : 0u;   // (uniform)
#pragma unroll
    for (int s = 0; s < G; ++s)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const u32x4 xv = xs[b][nb][s] & keep;
#pragma unroll
        for (int fr = 0; fr < FR; ++fr)
          acc[nb][fr] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ws[b][s][fr]),
                                                                __builtin_bit_cast(bf16x8, xv), acc[nb][fr], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
  };
  // wavefront w takes stages w PF .. w PF + PF - 1, then those 8 PF further on, ...: the PF stages it has in flight
  // are one contiguous run of every token row (PF KC values), which is what DRAM pages and cache lines like
  static_for<PF>([&](auto j) { load_stage(j, wave * PF + decltype(j)::value); });
  for (int c = wave * PF; c < n_stages; c += PF * GP_WAVES)
    static_for<PF>([&](auto j) {
      constexpr int jj = decltype(j)::value;
      multiply(j, c + jj);
      load_stage(j, c + jj + PF * GP_WAVES);
    });

  gate_finish<FR, NB>(acc, smem, t0, br, T, E, k, renorm, topk_idx, topk_w, probs);
}

template <int FR, int NB>
int32_t launch_packed(const moe_config* cfg, const void* x, const void* packed, const float* w_router, const float* b_router,
                      int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s) {
  constexpr int NT = 32 * NB, RW = 32 * FR, STRIDE = NT + 8;
  constexpr bool TWO_ROUNDS = (size_t)GP_WAVES * RW * STRIDE * 4 > 150 * 1024;
  constexpr size_t shmem = (size_t)(TWO_ROUNDS ? GP_WAVES / 2 : GP_WAVES) * RW * STRIDE * 4;
  static_assert(shmem <= 160 * 1024, "partial sums do not fit the LDS");
  auto kern = gate_packed_kernel<FR, NB>;
  if (shmem > 65536) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(gate LDS)");
  }
  hipLaunchKernelGGL(kern, dim3((cfg->T + NT - 1) / NT), dim3(GP_WAVES * 64), shmem, s, (const uint16_t*)x, (const uint16_t*)packed,
                     w_router, b_router, cfg->T, cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w, probs);
  hipLaunchKernelGGL(gate_fix_kernel, dim3((cfg->T + FIX_TOKENS - 1) / FIX_TOKENS), dim3(GP_WAVES * 64), 0, s, (const uint16_t*)x,
                     w_router, b_router, cfg->T, cfg->d_model, cfg->E, cfg->k, cfg->renormalize, topk_idx, topk_w, probs);
  return check_hip(hipGetLastError(), "gate launch");
}

}  // namespace

// A step of one token: gate and dispatch tables from one kernel (bf16 activations: the layer then needs no
// dispatched copy of the token).
bool gate_dispatch_one_token_applies(const moe_config* cfg, const float* w_router) {
  return cfg->T == 1 && cfg->dtype == MOE_BF16 && gate_few_applies(cfg, w_router);
}
int32_t launch_gate_dispatch_one_token(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                                       int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, int32_t* a2r,
                                       int32_t* r2a, int32_t* clear8, hipStream_t s) {
  return launch_few<uint16_t>(cfg, x, w_router, b_router, topk_idx, topk_w, nullptr, s, counts, offsets, a2r, r2a, clear8);
}

int32_t launch_gate(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                    int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  if (gate_few_applies(cfg, w_router)) {
    if (cfg->dtype == MOE_BF16) return launch_few<uint16_t>(cfg, x, w_router, b_router, topk_idx, topk_w, probs, s);
    return launch_few<float>(cfg, x, w_router, b_router, topk_idx, topk_w, probs, s);
  }
  if (cfg->dtype == MOE_BF16 && cfg->E <= 64) {
    if (cfg->E <= 16) return launch_fast<1>(cfg, x, w_router, b_router, topk_idx, topk_w, probs, s);
    if (cfg->E <= 32) return launch_fast<2>(cfg, x, w_router, b_router, topk_idx, topk_w, probs, s);
    return launch_fast<4>(cfg, x, w_router, b_router, topk_idx, topk_w, probs, s);
  }
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

// The pre-split router serves bfloat16 activations and up to 64 experts (3 E rows in at most six blocks of 32).
size_t router_pack_bytes(int d_model, int E) {
  if (E < 1 || E > 64 || d_model < 64 || d_model % 64) return 0;
  return (size_t)d_model * gate_frags(E) * 64;   // d/KC stages x G sub-steps x FR blocks x 1 KB
}

bool gate_packed_applies(const moe_config* cfg, const float* w_router) {
  return cfg->dtype == MOE_BF16 && cfg->E <= 64 && !gate_few_applies(cfg, w_router);
}
// Inside a layer the packed router is used where it measured faster than splitting on the fly: long token streams
// (from about 64 M activation elements; below, the kernels are bound by their chain of dependent steps and by the
// second launch that recomputes the near-ties, not by the split) and wide routers (more than 42 experts: there
// the split, which every workgroup repeats for the whole router, is most of the other kernel's time).
bool gate_packed_pays(const moe_config* cfg) {
  return (int64_t)cfg->T * cfg->d_model >= ((int64_t)1 << 26) || (gate_frags(cfg->E) >= 4 && cfg->T >= 1024);
}

int32_t launch_gate_packed(const moe_config* cfg, const void* x, const void* packed, const float* w_router, const float* b_router,
                           int32_t* topk_idx, float* topk_w, float* probs, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  const int FR = gate_frags(cfg->E);
  // tokens per workgroup: as many 32-token blocks as still give every compute unit a workgroup (each workgroup
  // reads the whole packed router once, from L2)
  const int forced = tuning(MOE_TUNE_GATE_TOKENS);
  auto wgs = [&](int nb) { return forced ? (forced == 32 * nb ? 1 << 20 : 0) : (cfg->T + 32 * nb - 1) / (32 * nb); };
#define MOE_GATE_PACKED(fr, nb) return launch_packed<fr, nb>(cfg, x, packed, w_router, b_router, topk_idx, topk_w, probs, s)
  switch (FR) {
    case 1:
      if (wgs(4) >= 256) MOE_GATE_PACKED(1, 4);
      if (wgs(2) >= 256) MOE_GATE_PACKED(1, 2);
      MOE_GATE_PACKED(1, 1);
    case 2:
      if (wgs(2) >= 256) MOE_GATE_PACKED(2, 2);
      MOE_GATE_PACKED(2, 1);
    case 3: MOE_GATE_PACKED(3, 1);
    case 4: MOE_GATE_PACKED(4, 1);
    case 5: MOE_GATE_PACKED(5, 1);
    case 6: MOE_GATE_PACKED(6, 1);
  }
#undef MOE_GATE_PACKED
  return fail(MOE_ERR_UNSUPPORTED, "packed router: E=%d has no kernel", cfg->E);
}

// The gate of a layer: on the pre-split router when the weights carry one and it applies.
int32_t launch_gate_of(const moe_config* cfg, const moe_weights* w, const void* x, int32_t* topk_idx, float* topk_w, float* probs,
                       hipStream_t s) {
  if (w->w_router_packed && gate_packed_applies(cfg, w->w_router) && gate_packed_pays(cfg))
    return launch_gate_packed(cfg, x, w->w_router_packed, w->w_router, w->b_router, topk_idx, topk_w, probs, s);
  return launch_gate(cfg, x, w->w_router, w->b_router, topk_idx, topk_w, probs, s);
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

extern "C" size_t moe_router_pack_bytes(int32_t d_model, int32_t E) { return router_pack_bytes(d_model, E); }

extern "C" int32_t moe_pack_router(const float* w_router, void* packed, int32_t d_model, int32_t E, void* stream) {
  const size_t bytes = router_pack_bytes(d_model, E);
  if (!bytes) return fail(MOE_ERR_UNSUPPORTED, "moe_pack_router: d_model=%d (multiple of 64) and E=%d (1..64) only", d_model, E);
  if (!w_router || !packed || ((uintptr_t)packed & 15)) return fail(MOE_ERR_INVALID_ARG, "moe_pack_router: NULL or misaligned pointer");
  const int FR = gate_frags(E), G = gate_substeps(FR);
  const size_t pieces = bytes / 16;
  hipLaunchKernelGGL(pack_router_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, (hipStream_t)stream, w_router,
                     (uint16_t*)packed, d_model, E, FR, G);
  return check_hip(hipGetLastError(), "router pack launch");
}

extern "C" int32_t moe_gate_packed(const moe_config* cfg, const void* x, const float* w_router, const float* b_router,
                                   const void* w_router_packed, int32_t* topk_idx, float* topk_w, float* probs, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (cfg->T > 0 && (!x || !w_router || !w_router_packed || !topk_idx || !topk_w))
    return fail(MOE_ERR_INVALID_ARG, "moe_gate_packed: x, w_router, w_router_packed, topk_idx and topk_w must be non-NULL");
  if (cfg->dtype != MOE_BF16 || cfg->E > 64)
    return fail(MOE_ERR_UNSUPPORTED, "moe_gate_packed: bf16 activations and at most 64 experts (use moe_gate)");
  if (!gate_packed_applies(cfg, w_router))   // steps of very few tokens: one workgroup per token on the float32 router
    return launch_gate(cfg, x, w_router, b_router, topk_idx, topk_w, probs, (hipStream_t)stream);
  return launch_gate_packed(cfg, x, w_router_packed, w_router, b_router, topk_idx, topk_w, probs, (hipStream_t)stream);
}
