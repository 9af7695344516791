// Grouped bf16 GEMM over variable per-expert row counts with fused epilogues:
// the expert FFN of the MoE layer (the sparsely activated FFN of Section 3.2).
//
//   GEMM1 (GELU)  : h[r, n]  = gelu(sum_k xd[r,k] * W1_e[n,k] + b1_e[n])
//   GEMM1 (SwiGLU): h[r, n]  = silu(sum_k xd[r,k] * Wg_e[n,k]) * (sum_k xd[r,k] * Wu_e[n,k])
//   GEMM2         : yd[r, n] = sum_k h[r,k] * W2_e[n,k] + b2_e[n]
// for r in [offsets[e], offsets[e+1]).  Both operands are K-contiguous
// (activations row-major, weights OUTPUT_MAJOR), accumulation is fp32 on the
// MFMA units, one rounding to bf16 at the end.
//
// CDNA4 mapping.  A workgroup owns a TOK x FEAT output tile and walks K in
// steps of 64.  Operand tiles go from global memory straight into LDS
// (global_load_lds_dwordx4, no register staging) as rows of 64 bf16 (128 B)
// whose eight 16-byte chunks are XOR-swizzled with the row index, so the
// per-lane 16-byte fragment reads of v_mfma_f32_32x32x16_bf16 spread over all
// banks; two stages alternate so that the next K-step streams in while the
// current one is multiplied.  The MFMA "A" operand is the weight fragment and the "B" operand the
// activation fragment: the accumulator then holds, per lane, one token and
// runs of four consecutive output features, which store as packed 8-byte
// pieces.  Tiles are enumerated on the device from expert_offsets (no host
// round trip), and consecutive tile ids are folded so that the workgroups that
// land on one XCD share operand tiles in that XCD's L2.
#include "moesys_internal.h"

namespace moesys {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int KSTEP = 64;          // K elements per LDS stage
constexpr int ROW_BYTES = KSTEP * 2;
constexpr int NUM_XCD = 8;

enum Epi { EPI_GELU = 0, EPI_SWIGLU = 1, EPI_BIAS = 2 };

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);  // v_cvt_pk_bf16_f32: round to nearest even
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float gelu_exact(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float silu(float u) { return u / (1.f + __expf(-u)); }

// LDS tile layout: row r (64 bf16 = 128 B) keeps its logical 16-byte chunk c at physical chunk
// c ^ ((r >> 1) & 7).  The LDS serves 16 lanes x 16 B per clock over 256 B of banks; with this key any 16
// consecutive rows read at one logical chunk hit 16 distinct 16-byte bank groups (measured conflict-free).

struct TileInfo {
  int expert, row0, rows;  // first dispatched row and valid rows (<= TOK) of this tile
  int ntile;               // feature tile index
};

// Maps blockIdx.x to a tile.  Returns false if this workgroup has nothing to do.
template <int TOK>
__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int E, int n_tiles, int* s_pref,
                                          TileInfo& ti) {
  // s_pref[e] = number of token tiles of experts < e ; s_pref[E] = total
  for (int e = threadIdx.x; e < E; e += blockDim.x) s_pref[e + 1] = (offsets[e + 1] - offsets[e] + TOK - 1) / TOK;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    s_pref[0] = 0;
    for (int e = 0; e < E; ++e) {
      run += s_pref[e + 1];
      s_pref[e + 1] = run;
    }
  }
  __syncthreads();
  const int total = s_pref[E] * n_tiles;
  const int chunk = (total + NUM_XCD - 1) / NUM_XCD;
  const int xcd = blockIdx.x % NUM_XCD, local = blockIdx.x / NUM_XCD;
  const int L = xcd * chunk + local;
  if (local >= chunk || L >= total) return false;
  const int mt = L / n_tiles;
  ti.ntile = L - mt * n_tiles;
  int lo = 0, hi = E;  // largest e with s_pref[e] <= mt
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (s_pref[mid] <= mt) lo = mid; else hi = mid;
  }
  // every lane computed the same values; say so to the compiler (they feed scalar descriptors)
  lo = __builtin_amdgcn_readfirstlane(lo);
  ti.expert = lo;
  const int r0 = __builtin_amdgcn_readfirstlane(offsets[lo] + (mt - s_pref[lo]) * TOK);
  ti.row0 = r0;
  ti.rows = __builtin_amdgcn_readfirstlane(min(TOK, offsets[lo + 1] - r0));
  ti.ntile = __builtin_amdgcn_readfirstlane(ti.ntile);
  return true;
}

// Raw buffer descriptor over [base, base+bytes): loads past the end return zero without touching memory,
// which is how rows beyond an expert's last row are masked.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
#endif

// TOK x FEAT tile, WT x WF wavefronts; each wavefront owns (TOK/WT) tokens x (FEAT/WF) LDS feature rows.
template <int TOK, int FEAT, int WT, int WF, int EPI>
__global__ __launch_bounds__(WT * WF * 64) void grouped_gemm_kernel(
    const uint16_t* __restrict__ act,     // [R, K]
    const uint16_t* __restrict__ wa,      // [E, N, K]   (W1 / Wg / W2)
    const uint16_t* __restrict__ wb,      // [E, N, K]   (Wu, SwiGLU only)
    const uint16_t* __restrict__ bias,    // [E, N] or NULL
    const int32_t* __restrict__ offsets,  // [E+1]
    uint16_t* __restrict__ out,           // [R, N]
    int E, int N, int K) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (buffer descriptors are device-only types)
  constexpr int NW = WT * WF;
  constexpr int WTOK = TOK / WT, WFEAT = FEAT / WF;
  constexpr int TB = WTOK / 32, FB = WFEAT / 32;  // 32x32 MFMA blocks per wavefront
  constexpr int A_BYTES = TOK * ROW_BYTES, B_BYTES = FEAT * ROW_BYTES;
  // SwiGLU: LDS feature rows [0,FEAT/2) come from Wg, [FEAT/2,FEAT) from Wu, for FEAT/2 output features
  constexpr int OUT_FEAT = EPI == EPI_SWIGLU ? FEAT / 2 : FEAT;
  constexpr int B_ROWS = OUT_FEAT;                                   // rows per weight matrix per tile
  constexpr int A_LOADS = TOK / 8 / NW, B_LOADS = B_ROWS / 8 / NW;   // wave-instructions per wavefront per stage
  static_assert(TOK % (8 * NW) == 0 && B_ROWS % (8 * NW) == 0, "tile/wavefront mismatch");
  static_assert(EPI != EPI_SWIGLU || FB == 2, "SwiGLU wave tile is one gate block + one up block");

  // two stages, as separate arrays so that the compiler can tell the stage being filled by LDS DMA from
  // the stage being read
  __shared__ __attribute__((aligned(1024))) unsigned char sA0[A_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sB0[B_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sA1[A_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char sB1[B_BYTES];
  __shared__ int s_pref[MOE_MAX_EXPERTS + 1];

  TileInfo ti;
  const int n_tiles = N / OUT_FEAT;
  if (!find_tile<TOK>(offsets, E, n_tiles, s_pref, ti)) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave / WF, wf = wave % WF;
  const int feat0 = ti.ntile * OUT_FEAT;
  const uint32_t row_bytes = (uint32_t)K * 2u;

  // ---- buffer descriptors and per-lane offsets of every direct-to-LDS load ---------------------
  const uint16_t* a_base_ptr = act + (size_t)ti.row0 * K;
  const uint16_t* b_base_ptr = wa + ((size_t)ti.expert * N + feat0) * K;
  const uint16_t* b2_base_ptr = (EPI == EPI_SWIGLU ? wb : wa) + ((size_t)ti.expert * N + feat0) * K;
  const uint32_t a_bytes = (uint32_t)ti.rows * row_bytes, b_bytes = (uint32_t)B_ROWS * row_bytes;
  int a_voff[A_LOADS], b_voff[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int r = (i * NW + wave) * 8 + (lane >> 3);
    a_voff[i] = r * (int)row_bytes + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int r = (i * NW + wave) * 8 + (lane >> 3);
    b_voff[i] = r * (int)row_bytes + (((lane & 7) ^ ((r >> 1) & 7)) << 4);
  }
  // One instruction moves 64 lanes x 16 B = eight 128-byte rows of a tile; lane l lands at row (l>>3),
  // physical chunk (l&7), and voff addresses the logical chunk that the swizzle maps there.  The K-step is
  // selected by the uniform offset.  `live` = false turns the stage into no-ops (zero-length descriptors).
#define MOE_TILE_LOADS(rsrc, voff, n_loads, lds_tile)                                                            \
  _Pragma("unroll") for (int i_ = 0; i_ < (n_loads); ++i_)                                                       \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                                  \
          rsrc, (__attribute__((address_space(3))) void*)((lds_tile) + (i_ * NW + wave) * 1024), 16, voff[i_], koff, 0, 0)
  auto issue_stage = [&](int kt, bool live, unsigned char* A, unsigned char* B) {
    const int koff = kt * ROW_BYTES;
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(a_base_ptr, live ? a_bytes : 0u);
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(b_base_ptr, live ? b_bytes : 0u);
    MOE_TILE_LOADS(a_rsrc, a_voff, A_LOADS, A);
    MOE_TILE_LOADS(b_rsrc, b_voff, B_LOADS, B);
    if (EPI == EPI_SWIGLU) {
      const __amdgpu_buffer_rsrc_t b2_rsrc = make_rsrc(b2_base_ptr, live ? b_bytes : 0u);
      MOE_TILE_LOADS(b2_rsrc, b_voff, B_LOADS, B + B_ROWS * ROW_BYTES);
    }
  };
#undef MOE_TILE_LOADS

  f32x16 acc[TB][FB];
#pragma unroll
  for (int i = 0; i < TB; ++i)
#pragma unroll
    for (int j = 0; j < FB; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // LDS byte address of this lane's fragment row with chunk key folded in: chunk for K sub-step ks is
  // (2*ks + half) ^ key = ((half ^ key) ^ 2*ks), i.e. base ^ (ks << 5).
  const int frow = lane & 31, fhalf = lane >> 5;
  int a_base[TB], w_base[FB];
#pragma unroll
  for (int i = 0; i < TB; ++i) {
    const int r = wt * WTOK + i * 32 + frow;
    a_base[i] = r * ROW_BYTES + ((fhalf ^ ((r >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int j = 0; j < FB; ++j) {
    int r;
    if (EPI == EPI_SWIGLU) r = j * (FEAT / 2) + wf * 32 + frow;  // j=0 gate rows, j=1 up rows
    else r = wf * WFEAT + j * 32 + frow;
    w_base[j] = r * ROW_BYTES + ((fhalf ^ ((r >> 1) & 7)) << 4);
  }

  auto read_frags = [&](const unsigned char* A, const unsigned char* B, int ks, bf16x8 (&af)[TB], bf16x8 (&wfr)[FB]) {
#pragma unroll
    for (int i = 0; i < TB; ++i) af[i] = *reinterpret_cast<const bf16x8*>(A + (a_base[i] ^ (ks << 5)));
#pragma unroll
    for (int j = 0; j < FB; ++j) wfr[j] = *reinterpret_cast<const bf16x8*>(B + (w_base[j] ^ (ks << 5)));
  };
  auto mfma_all = [&](const bf16x8 (&af)[TB], const bf16x8 (&wfr)[FB]) {
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[j], af[i], acc[i][j], 0, 0, 0);
  };
  // Asks the scheduler to alternate one MFMA with one LDS read (n pairs), then `tail` MFMAs.
  auto interleave = [&](int) {
#pragma unroll
    for (int q = 0; q < TB + FB; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
    }
    __builtin_amdgcn_sched_group_barrier(0x008, TB * FB - (TB + FB), 0);
  };

  // One K-step.  On entry fr[0] holds the fragments of sub-step 0 of the current stage (CA, CB), and the
  // loads of the next stage (NA, NB) were issued one K-step ago.  Sub-steps 0..2 multiply while the next
  // sub-step's fragments are read; then one barrier (all reads of the current stage done, next stage
  // landed); the current stage's buffers are refilled with stage kt+2 and the last sub-step multiplies
  // while sub-step 0 of the next stage is read.
  bf16x8 af[2][TB], wfr[2][FB];
  const int KT = K / KSTEP;
  auto step = [&](int kt, unsigned char* CA, unsigned char* CB, unsigned char* NA, unsigned char* NB) {
    read_frags(CA, CB, 1, af[1], wfr[1]);
    mfma_all(af[0], wfr[0]);
    interleave(0);
    read_frags(CA, CB, 2, af[0], wfr[0]);
    mfma_all(af[1], wfr[1]);
    interleave(0);
    read_frags(CA, CB, 3, af[1], wfr[1]);
    mfma_all(af[0], wfr[0]);
    interleave(0);
    __syncthreads();
    issue_stage(kt + 2, kt + 2 < KT, CA, CB);
    read_frags(NA, NB, 0, af[0], wfr[0]);
    mfma_all(af[1], wfr[1]);
    interleave(0);
  };

  issue_stage(0, true, sA0, sB0);
  __syncthreads();
  issue_stage(1, 1 < KT, sA1, sB1);
  read_frags(sA0, sB0, 0, af[0], wfr[0]);
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    step(kt, sA0, sB0, sA1, sB1);
    step(kt + 1, sA1, sB1, sA0, sB0);
  }
  if (kt < KT) step(kt, sA0, sB0, sA1, sB1);
  __syncthreads();  // no LDS DMA may be in flight past this point (the last stages issued were no-ops)

  // ---- epilogue: lane holds token (lane&31), features 8*i + 4*(lane>>5) + r of each 32x32 block ----
#pragma unroll
  for (int tb = 0; tb < TB; ++tb) {
    const int trow = wt * WTOK + tb * 32 + frow;
    if (trow >= ti.rows) continue;
    uint16_t* orow = out + (size_t)(ti.row0 + trow) * N;
    if (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = feat0 + wf * 32 + 8 * i + 4 * fhalf;
        uint32_t p[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) p[r] = f32_to_bf16_bits(silu(acc[tb][0][4 * i + r]) * acc[tb][1][4 * i + r]);
        u32x2 v;
        v.x = p[0] | (p[1] << 16);
        v.y = p[2] | (p[3] << 16);
        *reinterpret_cast<u32x2*>(orow + n) = v;
      }
    } else {
#pragma unroll
      for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int n = feat0 + wf * WFEAT + fb * 32 + 8 * i + 4 * fhalf;
          float bv[4] = {0.f, 0.f, 0.f, 0.f};
          if (bias) {
            const u32x2 b = *reinterpret_cast<const u32x2*>(bias + (size_t)ti.expert * N + n);
            bv[0] = bf16_bits_to_f32(b.x & 0xffffu); bv[1] = bf16_bits_to_f32(b.x >> 16);
            bv[2] = bf16_bits_to_f32(b.y & 0xffffu); bv[3] = bf16_bits_to_f32(b.y >> 16);
          }
          uint32_t p[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float u = acc[tb][fb][4 * i + r] + bv[r];
            if (EPI == EPI_GELU) u = gelu_exact(u);
            p[r] = f32_to_bf16_bits(u);
          }
          u32x2 v;
          v.x = p[0] | (p[1] << 16);
          v.y = p[2] | (p[3] << 16);
          *reinterpret_cast<u32x2*>(orow + n) = v;
        }
    }
  }
#endif
}

template <int TOK, int FEAT, int WT, int WF, int EPI>
int32_t launch(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb,
               const uint16_t* bias, const int32_t* offsets, uint16_t* out, int N, int K, hipStream_t s) {
  constexpr int OUT_FEAT = EPI == EPI_SWIGLU ? FEAT / 2 : FEAT;
  if (N % OUT_FEAT) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: N=%d is not a multiple of %d", N, OUT_FEAT);
  if (K % KSTEP) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d is not a multiple of %d", K, KSTEP);
  const int64_t rmax = max_rows(cfg);
  if (rmax == 0) return MOE_OK;
  int64_t mt = rmax / TOK + cfg->E;  // every expert may end in one partial tile
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS) {
    const int64_t by_cap = (int64_t)cfg->E * ((C + TOK - 1) / TOK);
    if (by_cap < mt) mt = by_cap;
  }
  int64_t total = mt * (N / OUT_FEAT);
  total = (total + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
  if (total > INT32_MAX) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: too many tiles");
  auto kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, EPI>;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(WT * WF * 64), 0, s, act, wa, wb, bias, offsets, out,
                     cfg->E, N, K);
  return check_hip(hipGetLastError(), "grouped GEMM launch");
}

}  // namespace

// Tile choice: 256x256 (8 wavefronts) when the feature count allows, else a 128-token tile with 64
// output features (4 wavefronts) so that any multiple of 64 is served.
int32_t launch_gemm1_bf16(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                          void* h, hipStream_t s) {
  const uint16_t* a = (const uint16_t*)xd;
  uint16_t* o = (uint16_t*)h;
  const int N = cfg->d_ff, K = cfg->d_model;
  if (cfg->act == MOE_ACT_SWIGLU) {
    const uint16_t *wg = (const uint16_t*)w->w_gate_proj, *wu = (const uint16_t*)w->w_up;
    if (N % 128 == 0) return launch<256, 256, 2, 4, EPI_SWIGLU>(cfg, a, wg, wu, nullptr, offsets, o, N, K, s);
    return launch<128, 128, 2, 2, EPI_SWIGLU>(cfg, a, wg, wu, nullptr, offsets, o, N, K, s);
  }
  const uint16_t *w1 = (const uint16_t*)w->w1, *b1 = (const uint16_t*)w->b1;
  if (N % 256 == 0) return launch<256, 256, 2, 4, EPI_GELU>(cfg, a, w1, nullptr, b1, offsets, o, N, K, s);
  return launch<128, 64, 4, 1, EPI_GELU>(cfg, a, w1, nullptr, b1, offsets, o, N, K, s);
}

int32_t launch_gemm2_bf16(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                          void* yd, hipStream_t s) {
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  const uint16_t* a = (const uint16_t*)h;
  const uint16_t* w2 = (const uint16_t*)(sw ? w->w_down : w->w2);
  const uint16_t* b2 = (const uint16_t*)(sw ? nullptr : w->b2);
  uint16_t* o = (uint16_t*)yd;
  const int N = cfg->d_model, K = cfg->d_ff;
  if (N % 256 == 0) return launch<256, 256, 2, 4, EPI_BIAS>(cfg, a, w2, nullptr, b2, offsets, o, N, K, s);
  return launch<128, 64, 4, 1, EPI_BIAS>(cfg, a, w2, nullptr, b2, offsets, o, N, K, s);
}

}  // namespace moesys
