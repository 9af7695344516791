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
// steps of KS (32 or 64).  Operand tiles go from global memory straight into
// LDS (buffer_load ... lds, 16 bytes per lane, no register staging) as rows of
// KS bf16 whose 16-byte chunks are XOR-swizzled with the row index, so that the
// per-lane 16-byte fragment reads of v_mfma_f32_32x32x16_bf16 are free of bank
// conflicts; two LDS stages alternate so that the next K-step streams in while
// the current one is multiplied, with ONE barrier per K-step placed before the
// step's last sub-step so that the first fragments of the next step are read
// under the tail of the current one.  The MFMA "A" operand is the weight
// fragment and the "B" operand the activation fragment: the accumulator then
// holds, per lane, one token and runs of four consecutive output features,
// which store as packed 8-byte pieces.  Rows past an expert's end are masked by
// the buffer descriptor (loads return zero, stores are skipped), never padded
// in memory.  Tiles are enumerated on the device from expert_offsets (no host
// round trip) in an order that makes the workgroups resident on one XCD share
// operand tiles in that XCD's L2, and the eight XCDs walk the same weight
// columns at the same time so that HBM serves each weight tile once.  When the
// last round of 256x256 tiles would occupy a minority of the CUs, those tiles
// are handed to a second launch that cuts each into four 256x64 tiles.
#include <cstdlib>
#include "moesys_internal.h"

namespace moesys {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int NUM_XCD = 8;
constexpr int CU_PER_XCD = 32;
constexpr int NUM_CU = NUM_XCD * CU_PER_XCD;
constexpr int BIG_FEAT = 256;       // feature width of the tile grid that orders the work
constexpr int SPLIT_MAX_LEFTOVER = 96;  // split the last round's tiles if there are at most this many
static_assert(SPLIT_MAX_LEFTOVER + 64 <= NUM_CU, "the narrow launch covers NUM_CU slots after the cut");

enum Epi { EPI_GELU = 0, EPI_SWIGLU = 1, EPI_BIAS = 2 };

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);  // v_cvt_pk_bf16_f32: round to nearest even
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// gelu(u) = u*Phi(u) = (u + |u| * erf(|u|/sqrt 2)) / 2 with erf from the five-term rational formula
// 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7): far below the bf16 rounding of h, at
// under half the instruction count of the library erff, which matters because this runs on every
// element of h while the matrix pipes wait.
__device__ __forceinline__ float gelu_fast(float u) {
  const float ax = fabsf(u) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(t, 1.061405429f, -1.453152027f);
  p = fmaf(t, p, 1.421413741f);
  p = fmaf(t, p, -0.284496736f);
  p = fmaf(t, p, 0.254829592f);
  p *= t;
  const float e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
  const float erf_abs = fmaf(-p, e, 1.0f);
  return 0.5f * fmaf(fabsf(u), erf_abs, u);
}
__device__ __forceinline__ float silu(float u) { return u * __builtin_amdgcn_rcpf(1.f + __expf(-u)); }

struct TileInfo {
  int expert, row0, rows;  // first dispatched row and valid rows (<= TOK) of this tile
  int ntile;               // feature tile index
};

// Tile order.  The work is ordered on a grid of TOK x 256 tiles.  Token tiles (of all experts, in row
// order) are grouped GM at a time and feature tiles GN at a time, GM*GN <= 32 = the workgroups one XCD
// starts together, so that an XCD's resident workgroups reuse GM activation tiles and GN weight tiles out
// of its L2.  The hardware hands workgroup i to XCD i mod 8; consecutive blocks b = 8q + xcd are laid out
// so that the eight XCDs work on eight token groups of the SAME feature group at the same time (one HBM
// read of those weights serves all of them through the shared cache level).  A trailing partial set of
// token groups is spread over the XCDs feature group by feature group instead, to keep them equally loaded.
//
// Slot i (the dispatch order) -> tile.  `cut` splits the slots between the two launches: if the tiles
// after the last full round of NUM_CU are few, the main launch stops at the cut and a second launch
// handles every later tile as SPLIT narrower tiles.  Both launches derive the cut from the same device
// data, so every tile is computed exactly once.
__host__ __device__ inline int group_n(int n_tiles) { return n_tiles < 8 ? n_tiles : 8; }
__host__ __device__ inline bool grid_is_dense(int n_tiles) {
  const int GN = group_n(n_tiles);
  return (CU_PER_XCD % GN) == 0 && (n_tiles % GN) == 0;
}

// SPLIT = 1: the main launch (blockIdx.x is the slot).  SPLIT > 1: the launch for the last round's tiles
// (blockIdx.x / SPLIT counts slots from the cut; blockIdx.x % SPLIT picks the narrow tile, in *sub).
template <int TOK, int SPLIT>
__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int E, int n_tiles, bool allow_split,
                                          int* s_pref, TileInfo& ti, int* sub) {
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
  const int MT = s_pref[E];
  const int total = MT * n_tiles;
  const int leftover = total % NUM_CU;
  const bool split_mode = allow_split && leftover > 0 && leftover <= SPLIT_MAX_LEFTOVER;
  const int cut = total - leftover;
  int slot;
  if (SPLIT == 1) {
    slot = blockIdx.x;
    if (split_mode && slot >= cut) return false;
  } else {
    if (!split_mode) return false;
    slot = cut + blockIdx.x / SPLIT;
    *sub = blockIdx.x % SPLIT;
  }
  const int GN = group_n(n_tiles), GM = CU_PER_XCD / GN;
  const int MG = (MT + GM - 1) / GM, NG = (n_tiles + GN - 1) / GN;
  const int xcd = slot % NUM_XCD, local = slot / NUM_XCD;
  const int q = local / CU_PER_XCD, t = local % CU_PER_XCD;
  const int b = q * NUM_XCD + xcd;
  if (t >= GM * GN || b >= MG * NG) return false;
  const int msg = b / (NUM_XCD * NG), rem = b - msg * NUM_XCD * NG;
  const int P = min(NUM_XCD, MG - msg * NUM_XCD);
  const int ng = rem / P, mg = msg * NUM_XCD + rem % P;
  const int mt = mg * GM + t / GN, nt = ng * GN + t % GN;
  if (mt >= MT || nt >= n_tiles) return false;
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
  ti.ntile = __builtin_amdgcn_readfirstlane(nt);
  return true;
}

// Raw buffer descriptor over [base, base+bytes): loads past the end return zero without touching memory,
// which is how rows beyond an expert's last row are masked.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
#endif

// TOK x FEAT tile, WT x WF wavefronts, K-step KS; each wavefront owns (TOK/WT) tokens x (FEAT/WF) LDS
// feature rows.  WPE = wavefronts per SIMD the register budget is sized for.  SPLIT = 1 for the main
// launch; SPLIT > 1 for the launch that cuts the last round's 256-wide tiles into SPLIT narrow ones.
template <int TOK, int FEAT, int WT, int WF, int KS, int NST, int WPE, int SPLIT, int EPI>
__global__ __launch_bounds__(WT * WF * 64, WPE) void grouped_gemm_kernel(
    const uint16_t* __restrict__ act,     // [R, K]
    const uint16_t* __restrict__ wa,      // [E, N, K]   (W1 / Wg / W2)
    const uint16_t* __restrict__ wb,      // [E, N, K]   (Wu, SwiGLU only)
    const uint16_t* __restrict__ bias,    // [E, N] or NULL
    const int32_t* __restrict__ offsets,  // [E+1]
    uint16_t* __restrict__ out,           // [R, N]
    int E, int N, int K, int allow_split) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (buffer descriptors are device-only types)
  constexpr int NW = WT * WF;
  constexpr int WTOK = TOK / WT, WFEAT = FEAT / WF;
  constexpr int TB = WTOK / 32, FB = WFEAT / 32;  // 32x32 MFMA blocks per wavefront
  constexpr int ROW_BYTES = KS * 2;               // one LDS row
  constexpr int CHUNKS = KS / 8;                  // 16-byte chunks per row
  constexpr int RPB = 256 / ROW_BYTES;            // rows per 256 bytes (the LDS bank period for 16-byte reads)
  constexpr int RPI = 1024 / ROW_BYTES;           // rows moved by one wave-wide 16-byte-per-lane load
  constexpr int NSUB = KS / 16;                   // MFMA sub-steps per K-step
  constexpr int A_BYTES = TOK * ROW_BYTES, B_BYTES = FEAT * ROW_BYTES;
  // SwiGLU: LDS feature rows [0,FEAT/2) come from Wg, [FEAT/2,FEAT) from Wu, for FEAT/2 output features
  constexpr int OUT_FEAT = EPI == EPI_SWIGLU ? FEAT / 2 : FEAT;
  constexpr int B_ROWS = OUT_FEAT;                                    // rows per weight matrix per tile
  constexpr int A_LOADS = TOK / RPI / NW, B_LOADS = B_ROWS / RPI / NW;  // wave-instructions per wavefront per stage
  // tiles are ordered on a grid whose feature width is GRID_FEAT; a SPLIT launch cuts each grid tile
  constexpr int GRID_FEAT = OUT_FEAT * SPLIT;
  static_assert(TOK % (RPI * NW) == 0 && B_ROWS % (RPI * NW) == 0, "tile/wavefront mismatch");
  static_assert(EPI != EPI_SWIGLU || FB == 2, "SwiGLU wave tile is one gate block + one up block");
  static_assert(NSUB == 2 || NSUB == 4, "K-step is 32 or 64");

  // LDS tile layout: row r keeps its logical 16-byte chunk c at physical chunk c ^ key(r), key(r) =
  // (r / RPB) mod CHUNKS.  The LDS serves 16 lanes x 16 B per clock over a 256-byte bank period; with this
  // key any 16 consecutive rows read at one logical chunk land on 16 distinct 16-byte bank groups
  // (measured conflict-free on gfx950, where keying on r mod 8 gives 2-way conflicts).
  // NST stages (2 or 4), each one array holding the token tile then the feature tile: separate arrays so
  // that the compiler can tell a stage being filled by LDS DMA from the stage being read.
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static_assert(NST == 2 || NST == 4, "two or four LDS stages");
  __shared__ __attribute__((aligned(1024))) unsigned char s0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char s1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char s2[NST == 4 ? STAGE_BYTES : 16];
  __shared__ __attribute__((aligned(1024))) unsigned char s3[NST == 4 ? STAGE_BYTES : 16];
  __shared__ int s_pref[MOE_MAX_EXPERTS + 1];

  TileInfo ti;
  int sub = 0;
  if (!find_tile<TOK, SPLIT>(offsets, E, N / GRID_FEAT, allow_split != 0, s_pref, ti, &sub)) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave / WF, wf = wave % WF;
  const int feat0 = ti.ntile * GRID_FEAT + __builtin_amdgcn_readfirstlane(sub) * OUT_FEAT;
  const uint32_t row_bytes = (uint32_t)K * 2u;

  // ---- buffer descriptors and per-lane offsets of every direct-to-LDS load ---------------------
  const uint16_t* a_base_ptr = act + (size_t)ti.row0 * K;
  const uint16_t* b_base_ptr = wa + ((size_t)ti.expert * N + feat0) * K;
  const uint16_t* b2_base_ptr = (EPI == EPI_SWIGLU ? wb : wa) + ((size_t)ti.expert * N + feat0) * K;
  const uint32_t a_bytes = (uint32_t)ti.rows * row_bytes, b_bytes = (uint32_t)B_ROWS * row_bytes;
  int a_voff[A_LOADS], b_voff[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int r = (i * NW + wave) * RPI + lane / CHUNKS;
    a_voff[i] = r * (int)row_bytes + (((lane % CHUNKS) ^ ((r / RPB) % CHUNKS)) << 4);
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int r = (i * NW + wave) * RPI + lane / CHUNKS;
    b_voff[i] = r * (int)row_bytes + (((lane % CHUNKS) ^ ((r / RPB) % CHUNKS)) << 4);
  }
  // One instruction moves 64 lanes x 16 B = RPI rows of a tile; lane l lands at row l/CHUNKS, physical
  // chunk l%CHUNKS, and voff addresses the logical chunk that the swizzle maps there.  The K-step is
  // selected by the uniform offset.  `live` = false turns the stage into no-ops (zero-length descriptors).
#define MOE_TILE_LOADS(rsrc, voff, n_loads, lds_tile)                                                            \
  _Pragma("unroll") for (int i_ = 0; i_ < (n_loads); ++i_)                                                       \
      __builtin_amdgcn_raw_ptr_buffer_load_lds(                                                                  \
          rsrc, (__attribute__((address_space(3))) void*)((lds_tile) + (i_ * NW + wave) * 1024), 16, voff[i_], koff, 0, 0)
  auto issue_stage = [&](int kt, bool live, unsigned char* stage) {
    unsigned char* A = stage;
    unsigned char* B = stage + A_BYTES;
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

  // LDS byte address of this lane's fragment row with chunk key folded in: the chunk of K sub-step ks is
  // (2*ks + half) ^ key = (half ^ key) ^ 2*ks, i.e. base ^ (ks << 5).
  const int frow = lane & 31, fhalf = lane >> 5;
  int a_base[TB], w_base[FB];
#pragma unroll
  for (int i = 0; i < TB; ++i) {
    const int r = wt * WTOK + i * 32 + frow;
    a_base[i] = r * ROW_BYTES + ((fhalf ^ ((r / RPB) % CHUNKS)) << 4);
  }
#pragma unroll
  for (int j = 0; j < FB; ++j) {
    int r;
    if (EPI == EPI_SWIGLU) r = j * (FEAT / 2) + wf * 32 + frow;  // j=0 gate rows, j=1 up rows
    else r = wf * WFEAT + j * 32 + frow;
    w_base[j] = r * ROW_BYTES + ((fhalf ^ ((r / RPB) % CHUNKS)) << 4);
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
  // Asks the scheduler to alternate one MFMA with one LDS read, then the remaining MFMAs.
  auto interleave = [&]() {
    constexpr int PAIRS = TB + FB < TB * FB ? TB + FB : TB * FB;
#pragma unroll
    for (int q = 0; q < PAIRS; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
    }
    if (TB * FB > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, TB * FB - PAIRS, 0);
  };

  // One K-step on the stage in `cur`.  On entry fr[0] holds the fragments of sub-step 0 of that stage and
  // the loads of the following NST-1 stages are in flight.  All sub-steps but the last multiply while the
  // next sub-step's fragments are read; then every wavefront waits until its own share of the NEXT stage
  // has landed (the younger NST-2 batches may stay in flight: the counter retires loads in order) and until
  // its fragment reads are done, and the workgroup meets at one barrier; the current stage's buffer is then
  // refilled with stage kt+NST, and the last sub-step multiplies while sub-step 0 of the next stage is read.
  constexpr int LOADS_PER_STAGE = A_LOADS + B_LOADS * (EPI == EPI_SWIGLU ? 2 : 1);
  constexpr int IN_FLIGHT = (NST - 2) * LOADS_PER_STAGE;  // loads allowed to be outstanding at the barrier
  static_assert(IN_FLIGHT < 64, "vmcnt is a 6-bit counter");
  // s_waitcnt immediate: vmcnt = IN_FLIGHT (bits 3:0 and 15:14), expcnt = 7 (no wait), lgkmcnt = 0
  constexpr int WAIT_IMM = (IN_FLIGHT & 15) | ((IN_FLIGHT >> 4) << 14) | (7 << 4);
  auto stage_barrier = [&]() {
    asm volatile("s_waitcnt %0\n\ts_barrier" ::"n"(WAIT_IMM) : "memory");
  };
  bf16x8 af[2][TB], wfr[2][FB];
  const int KT = K / KS;
  auto step = [&](int kt, unsigned char* cur, unsigned char* nxt) {
#pragma unroll
    for (int ks = 0; ks + 1 < NSUB; ++ks) {
      read_frags(cur, cur + A_BYTES, ks + 1, af[(ks + 1) & 1], wfr[(ks + 1) & 1]);
      mfma_all(af[ks & 1], wfr[ks & 1]);
      interleave();
    }
    stage_barrier();
    issue_stage(kt + NST, kt + NST < KT, cur);
    read_frags(nxt, nxt + A_BYTES, 0, af[0], wfr[0]);
    mfma_all(af[(NSUB - 1) & 1], wfr[(NSUB - 1) & 1]);
    interleave();
  };

  issue_stage(0, true, s0);
  issue_stage(1, 1 < KT, s1);
  if (NST == 4) {
    issue_stage(2, 2 < KT, s2);
    issue_stage(3, 3 < KT, s3);
  }
  {  // stage 0 has landed for every wavefront
    constexpr int PRO = (NST - 1) * LOADS_PER_STAGE;
    constexpr int PRO_IMM = (PRO & 15) | ((PRO >> 4) << 14) | (7 << 4);
    static_assert(PRO < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt %0\n\ts_barrier" ::"n"(PRO_IMM) : "memory");
  }
  read_frags(s0, s0 + A_BYTES, 0, af[0], wfr[0]);
  int kt = 0;
  if (NST == 2) {
    for (; kt + 1 < KT; kt += 2) {
      step(kt, s0, s1);
      step(kt + 1, s1, s0);
    }
    if (kt < KT) step(kt, s0, s1);
  } else {
    for (; kt + 3 < KT; kt += 4) {
      step(kt, s0, s1);
      step(kt + 1, s1, s2);
      step(kt + 2, s2, s3);
      step(kt + 3, s3, s0);
    }
    if (kt < KT) step(kt, s0, s1);
    if (kt + 1 < KT) step(kt + 1, s1, s2);
    if (kt + 2 < KT) step(kt + 2, s2, s3);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // only zero-length loads remain; retire them before exit

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
            if (EPI == EPI_GELU) u = gelu_fast(u);
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

template <int TOK, int FEAT, int WT, int WF, int KS, int NST, int WPE, int SPLIT, int EPI>
int32_t launch(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb,
               const uint16_t* bias, const int32_t* offsets, uint16_t* out, int N, int K, bool allow_split,
               hipStream_t s) {
  constexpr int OUT_FEAT = EPI == EPI_SWIGLU ? FEAT / 2 : FEAT;
  constexpr int GRID_FEAT = OUT_FEAT * SPLIT;
  if (N % GRID_FEAT) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: N=%d is not a multiple of %d", N, GRID_FEAT);
  if (K % KS) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d is not a multiple of %d", K, KS);
  if ((int64_t)TOK * K * 2 >= ((int64_t)1 << 31)) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d too large", K);
  const int64_t rmax = max_rows(cfg);
  if (rmax == 0) return MOE_OK;
  int64_t total;
  if (SPLIT == 1) {
    int64_t mt = rmax / TOK + cfg->E;  // every expert may end in one partial tile
    const int64_t C = moe_capacity(cfg);
    if (C != MOE_DROPLESS) {
      const int64_t by_cap = (int64_t)cfg->E * ((C + TOK - 1) / TOK);
      if (by_cap < mt) mt = by_cap;
    }
    const int n_tiles = N / GRID_FEAT;
    const int GN = group_n(n_tiles), GM = CU_PER_XCD / GN;
    const int64_t MG = (mt + GM - 1) / GM, NG = (n_tiles + GN - 1) / GN;
    total = (MG * NG + NUM_XCD - 1) / NUM_XCD * CU_PER_XCD * NUM_XCD;  // whole blocks on every XCD
  } else {
    // Slots from the cut to the last tile: the leftover tiles (<= SPLIT_MAX_LEFTOVER) plus the empty slots
    // of the last, partial token group (< GM * n_tiles <= 64 for the grids splitting is enabled on).
    total = (int64_t)NUM_CU * SPLIT;
  }
  if (total > INT32_MAX) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: too many tiles");
  auto kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, NST, WPE, SPLIT, EPI>;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(WT * WF * 64), 0, s, act, wa, wb, bias, offsets, out,
                     cfg->E, N, K, allow_split ? 1 : 0);
  return check_hip(hipGetLastError(), "grouped GEMM launch");
}

// MOESYS_GEMM_SPLIT=1 enables the narrow-tile launch for the last round.  Off by default: measured on
// MI355X the K loop of a narrow tile is bound by the same per-step memory latency as the wide tile's, so
// a quarter-width tile takes almost as long as a full one and the split loses.
bool split_enabled() {
  static const bool v = [] { const char* e = getenv("MOESYS_GEMM_SPLIT"); return e && atoi(e) != 0; }();
  return v;
}

// MOESYS_GEMM_DEEP=1 selects four 32-deep LDS stages instead of two 64-deep ones.  Off by default:
// measured ~7 % slower on MI355X (twice the barriers, no gain from the longer prefetch distance).
bool deep_pipeline() {
  static const bool v = [] { const char* e = getenv("MOESYS_GEMM_DEEP"); return e && atoi(e) != 0; }();
  return v;
}

// One grouped GEMM = the 256x256x64 launch (8 wavefronts, one workgroup per CU: the highest arithmetic
// intensity that fits the 160 KB LDS) plus, when the feature count lets the slot grid be dense, the
// narrow-tile launch for the last round.  Feature counts that are multiples of 64 but not of 256 use
// narrow tiles throughout.
// Token-tile height.  256 rows is the default; 320 rows (10 MFMA row blocks, still within the 160 KB LDS)
// is chosen when, for the row count an evenly loaded expert would get, it saves enough whole rounds of
// NUM_CU tiles to pay for the taller tile (e.g. ~1024 rows per expert: 4 tiles of 320 instead of 5 of 256).
// The estimate only steers the choice; any routing is handled by either height.
static int pick_tile_rows(const moe_config* cfg, int n_tiles) {
  static const int forced = [] { const char* e = getenv("MOESYS_GEMM_TOK"); return e ? atoi(e) : 0; }();
  if (forced == 256 || forced == 320) return forced;
  const int64_t A = (int64_t)cfg->k * cfg->T;
  int64_t rows = (A + cfg->E - 1) / cfg->E;
  rows += (rows * 2 + 24) / 25;  // 8 % head-room for uneven routing
  const int64_t C = moe_capacity(cfg);
  if (rows > C) rows = C;
  if (rows < 1) rows = 1;
  int best = 256;
  int64_t best_cost = -1;
  for (int tok : {256, 320}) {
    const int64_t tiles = (int64_t)cfg->E * ((rows + tok - 1) / tok) * n_tiles;
    const int64_t cost = (tiles + NUM_CU - 1) / NUM_CU * tok;
    if (best_cost < 0 || cost < best_cost) { best = tok; best_cost = cost; }
  }
  return best;
}

template <int EPI, int KSB, int NSB>
int32_t gemm_any(const moe_config* cfg, const uint16_t* a, const uint16_t* wa, const uint16_t* wb, const uint16_t* bias,
                 const int32_t* offsets, uint16_t* o, int N, int K, hipStream_t s) {
  constexpr int BF = EPI == EPI_SWIGLU ? 128 : 256;  // output features of the big tile
  if (N % BF == 0) {
    const bool sp = split_enabled() && grid_is_dense(N / BF) && N / BF <= 16;
    if (!sp && KSB == 64 && pick_tile_rows(cfg, N / BF) == 320)
      return launch<320, 256, 2, 4, 64, 2, 2, 1, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, false, s);
    int32_t st = launch<256, 256, 2, 4, KSB, NSB, 2, 1, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, sp, s);
    if (st != MOE_OK || !sp) return st;
    if constexpr (EPI == EPI_SWIGLU)  // 128 output features -> two tiles of 64 (gate rows + up rows side by side)
      return launch<256, 128, 4, 2, 64, 2, 2, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, true, s);
    else
      return launch<256, 64, 4, 2, 64, 2, 2, 4, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, true, s);
  }
  if constexpr (EPI == EPI_SWIGLU)
    return launch<128, 128, 2, 2, 64, 2, 2, 1, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, false, s);
  else
    return launch<128, 64, 4, 1, 64, 2, 2, 1, EPI>(cfg, a, wa, wb, bias, offsets, o, N, K, false, s);
}

}  // namespace

int32_t launch_gemm1_bf16(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                          void* h, hipStream_t s) {
  if (cfg->act == MOE_ACT_SWIGLU)
    return (deep_pipeline() ? gemm_any<EPI_SWIGLU, 32, 4> : gemm_any<EPI_SWIGLU, 64, 2>)(cfg, (const uint16_t*)xd, (const uint16_t*)w->w_gate_proj, (const uint16_t*)w->w_up,
                                nullptr, offsets, (uint16_t*)h, cfg->d_ff, cfg->d_model, s);
  return (deep_pipeline() ? gemm_any<EPI_GELU, 32, 4> : gemm_any<EPI_GELU, 64, 2>)(cfg, (const uint16_t*)xd, (const uint16_t*)w->w1, nullptr, (const uint16_t*)w->b1, offsets,
                            (uint16_t*)h, cfg->d_ff, cfg->d_model, s);
}

int32_t launch_gemm2_bf16(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                          void* yd, hipStream_t s) {
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  return (deep_pipeline() ? gemm_any<EPI_BIAS, 32, 4> : gemm_any<EPI_BIAS, 64, 2>)(cfg, (const uint16_t*)h, (const uint16_t*)(sw ? w->w_down : w->w2), nullptr,
                            (const uint16_t*)(sw ? nullptr : w->b2), offsets, (uint16_t*)yd, cfg->d_model, cfg->d_ff, s);
}

}  // namespace moesys
