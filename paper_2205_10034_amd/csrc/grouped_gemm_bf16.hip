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
// CDNA4 mapping.  The kernel is persistent: one workgroup per CU walks the
// tile list with a stride of the CU count.  A workgroup owns a TOK x FEAT
// output tile and walks K in steps of KS (32 or 64).  Operand tiles go from
// global memory straight into LDS (buffer_load ... lds, 16 bytes per lane, no
// register staging) as rows of KS bf16 whose 16-byte chunks are XOR-swizzled
// with the row index, so that the per-lane 16-byte fragment reads of
// v_mfma_f32_32x32x16_bf16 are free of bank conflicts; NST LDS stages rotate so
// that the next K-steps stream in while the current one is multiplied, with ONE
// barrier per K-step placed before the step's last sub-step so that the first
// fragments of the next step are read under the tail of the current one.  The
// first stages of the NEXT tile are requested before the epilogue of the
// current one, so their latency hides under the activation and the stores.
// The MFMA "A" operand is the weight fragment and the "B" operand the
// activation fragment: the accumulator then holds, per lane, one token and runs
// of four consecutive output features, which store as packed 8-byte pieces.
// Rows past an expert's end are masked by the buffer descriptor (loads return
// zero, stores are skipped), never padded in memory.  Tiles are enumerated on
// the device from expert_offsets (no host round trip) in an order that makes
// the workgroups resident on one XCD share operand tiles in that XCD's L2, and
// the eight XCDs walk the same weight columns at the same time so that HBM
// serves each weight tile once.
#include <cstdlib>
#include <type_traits>
#include "moesys_internal.h"

namespace moesys {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int NUM_XCD = 8;
constexpr int CU_PER_XCD = 32;
constexpr int NUM_CU = NUM_XCD * CU_PER_XCD;

enum Epi { EPI_GELU = 0, EPI_SWIGLU = 1, EPI_BIAS = 2 };

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);  // v_cvt_pk_bf16_f32: round to nearest even
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// gelu(u) = u * Phi(u).  Phi comes from a table in LDS: PHI_N entries (Phi(x_i), Phi(x_i+1) - Phi(x_i)) on
// x_i = -PHI_RANGE + i / PHI_SCALE, filled once per workgroup with the exact erf, and read with linear
// interpolation.  Interpolation error <= h^2/8 * max|Phi''| = (1/64)^2 / 8 * 0.242 = 7.4e-6, far below the
// bf16 rounding of h; outside the range Phi is 0 or 1 to 6e-16.  A table read plus ~9 ALU operations
// replaces ~50 for the library erff: the activation runs on every element of h while the matrix pipes
// wait, so its instruction count is what the GEMM1 epilogue costs.
constexpr int PHI_N = 1024;
constexpr float PHI_RANGE = 8.0f, PHI_SCALE = 64.0f;

__device__ __forceinline__ void fill_phi_table(f32x2* tab) {
  for (int i = threadIdx.x; i < PHI_N; i += blockDim.x) {
    const float x0 = -PHI_RANGE + (float)i / PHI_SCALE, x1 = -PHI_RANGE + (float)(i + 1) / PHI_SCALE;
    const float p0 = 0.5f * erfcf(-x0 * 0.70710678118654752f), p1 = 0.5f * erfcf(-x1 * 0.70710678118654752f);
    tab[i] = f32x2{p0, p1 - p0};
  }
}
__device__ __forceinline__ float gelu_table(float u, const f32x2* tab) {
  float t = fmaf(u, PHI_SCALE, PHI_RANGE * PHI_SCALE);
  t = __builtin_amdgcn_fmed3f(t, 0.0f, (float)PHI_N - 0.001f);
  const int i = (int)t;
  const f32x2 e = tab[i];
  return u * fmaf(t - (float)i, e.y, e.x);
}
__device__ __forceinline__ float silu(float u) { return u * __builtin_amdgcn_rcpf(1.f + __expf(-u)); }

struct TileInfo {
  int expert, row0, rows;  // first dispatched row and valid rows (<= TOK) of this tile
  int ntile;               // feature tile index
};

// Tile order.  Token tiles (of all experts, in row order) are grouped GM at a time and feature tiles GN
// at a time, GM*GN <= 32 = the CUs of one XCD, so that an XCD's workgroups reuse GM activation tiles and
// GN weight tiles out of its L2.  Workgroup w (on XCD w mod 8: the hardware hands workgroups to XCDs round
// robin) works on blocks b = 8q + xcd of up to 32 tiles, which are laid out so that
// the eight XCDs work on eight token groups of the SAME feature group at the same time (one HBM read of
// those weights serves all of them through the shared cache level).  A trailing partial set of token
// groups is spread over the XCDs feature group by feature group instead, to keep them equally loaded.
__host__ __device__ inline int group_n(int n_tiles) { return n_tiles < 8 ? n_tiles : 8; }

// s_pref[e] = number of token tiles of experts < e ; s_pref[E] = total.  Whole workgroup.
template <int TOK>
__device__ __forceinline__ void count_token_tiles(const int32_t* __restrict__ offsets, int E, int* s_pref) {
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
}

// Upper bound (host) of the number of blocks of up to 32 tiles.
__host__ __device__ inline int64_t block_count(int64_t MT, int n_tiles) {
  const int GN = group_n(n_tiles), GM = CU_PER_XCD / GN;
  return ((MT + GM - 1) / GM) * ((n_tiles + GN - 1) / GN);
}

// Walks the tiles of one workgroup.  Block b (b mod 8 = the XCD) holds the gm x gn tiles of token group mg
// and feature group ng (partial groups hold fewer).  The workgroups of an XCD share that XCD's blocks:
// the tiles of blocks x, x+8, x+16, ... are numbered consecutively and workgroup j of the G on the XCD
// takes numbers j, j+G, j+2G, ... - a fixed, gap-free assignment with no counters and no atomics.
template <int TOK>
struct TileWalker {
  int MT, NT, GM, GN, MG, NG;
  int xcd, G;
  int q, base, want;

  __device__ __forceinline__ void init(int mt_total, int n_tiles) {
    MT = mt_total; NT = n_tiles;
    GN = group_n(n_tiles); GM = CU_PER_XCD / GN;
    MG = (MT + GM - 1) / GM; NG = (NT + GN - 1) / GN;
    xcd = blockIdx.x % NUM_XCD; G = gridDim.x / NUM_XCD;
    q = 0; base = 0; want = blockIdx.x / NUM_XCD;
  }
  // Next tile of this workgroup; false when there is none.  All values are wave-uniform.
  __device__ __forceinline__ bool next(const int32_t* __restrict__ offsets, int E, const int* s_pref, TileInfo& ti) {
    const int n_blocks = MG * NG;
    while (true) {
      const int b = q * NUM_XCD + xcd;
      if (b >= n_blocks) return false;
      const int msg = b / (NUM_XCD * NG), rem = b - msg * NUM_XCD * NG;
      const int P = min(NUM_XCD, MG - msg * NUM_XCD);
      const int ng = rem / P, mg = msg * NUM_XCD + rem % P;
      const int gm = min(GM, MT - mg * GM), gn = min(GN, NT - ng * GN);
      const int cnt = gm * gn;
      if (want < base + cnt) {
        const int r = want - base;
        const int mt = mg * GM + r / gn, nt = ng * GN + r % gn;
        want += G;
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
      base += cnt;
      ++q;
    }
  }
};

// Raw buffer descriptor over [base, base+bytes): loads past the end return zero without touching memory,
// which is how rows beyond an expert's last row are masked.
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
#endif

// TOK x FEAT tile, WT x WF wavefronts, K-step KS, NST LDS stages; each wavefront owns (TOK/WT) tokens x
// (FEAT/WF) LDS feature rows.  WPE = wavefronts per SIMD the register budget is sized for.
template <int TOK, int FEAT, int WT, int WF, int KS, int NST, int WPE, int EPI, bool GATHER>
__global__ __launch_bounds__(WT * WF * 64, WPE) void grouped_gemm_kernel(
    const uint16_t* __restrict__ act,     // [R, K]
    const uint16_t* __restrict__ wa,      // [E, N, K]   (W1 / Wg / W2)
    const uint16_t* __restrict__ wb,      // [E, N, K]   (Wu, SwiGLU only)
    const uint16_t* __restrict__ bias,    // [E, N] or NULL
    const int32_t* __restrict__ offsets,  // [E+1]
    uint16_t* __restrict__ out,           // [R, N]
    const int32_t* __restrict__ row_map,  // GATHER: row_to_assign; act is then x[T,K] and row r reads token row_map[r] mod T
    int T, int E, int N, int K) {
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
  __shared__ f32x2 s_phi[EPI == EPI_GELU ? PHI_N : 1];
  __shared__ int s_pref[MOE_MAX_EXPERTS + 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave / WF, wf = wave % WF;
  const uint32_t row_bytes = (uint32_t)K * 2u;
  const int n_tiles = N / OUT_FEAT;

  if (EPI == EPI_GELU) fill_phi_table(s_phi);
  count_token_tiles<TOK>(offsets, E, s_pref);  // ends with a barrier: s_pref and the table are visible
  TileWalker<TOK> walk;
  walk.init(s_pref[E], n_tiles);

  // ---- per-lane offsets of every direct-to-LDS load, LDS fragment addresses ----------------------
  // (with a row map the token-tile offsets are recomputed per tile from the gathered token indices)
  int a_voff[A_LOADS], b_voff[B_LOADS];
  // byte offset of this lane's chunk inside its row, swizzle applied
  auto a_chunk = [&](int i) {
    const int r = (i * NW + wave) * RPI + lane / CHUNKS;
    return ((lane % CHUNKS) ^ ((r / RPB) % CHUNKS)) << 4;
  };
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int r = (i * NW + wave) * RPI + lane / CHUNKS;
    a_voff[i] = r * (int)row_bytes + a_chunk(i);
  }
  // token index of each of this lane's token-tile rows (-1 past the tile's last row)
  auto fetch_rows = [&](const TileInfo& t, int (&tok)[GATHER ? A_LOADS : 1]) {
#pragma unroll
    for (int i = 0; i < (GATHER ? A_LOADS : 1); ++i) {
      const int r = (i * NW + wave) * RPI + lane / CHUNKS;
      tok[i] = r < t.rows ? row_map[t.row0 + r] : -1;
    }
  };
  auto gather_voff = [&](const int (&tok)[GATHER ? A_LOADS : 1]) {
#pragma unroll
    for (int i = 0; i < (GATHER ? A_LOADS : 1); ++i) {
      int t = tok[i];
      while (t >= T) t -= T;  // assignment id j*T + t -> token (j < k <= 8)
      a_voff[i] = t >= 0 ? t * (int)row_bytes + a_chunk(i) : 0x7fffffff;  // past the end of x: reads zero
    }
  };
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int r = (i * NW + wave) * RPI + lane / CHUNKS;
    b_voff[i] = r * (int)row_bytes + (((lane % CHUNKS) ^ ((r / RPB) % CHUNKS)) << 4);
  }
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

  // ---- the current tile's operand windows (wave-uniform) ----------------------------------------
  const uint16_t *a_ptr = act, *b_ptr = wa, *b2_ptr = wa;
  uint32_t a_bytes = 0;
  const uint32_t b_bytes = (uint32_t)B_ROWS * row_bytes;
  auto bind_tile = [&](const TileInfo& t) {
    const size_t woff = ((size_t)t.expert * N + (size_t)t.ntile * OUT_FEAT) * K;
    a_ptr = GATHER ? act : act + (size_t)t.row0 * K;
    b_ptr = wa + woff;
    b2_ptr = (EPI == EPI_SWIGLU ? wb : wa) + woff;
    a_bytes = (GATHER ? (uint32_t)T : (uint32_t)t.rows) * row_bytes;
  };
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
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(a_ptr, live ? a_bytes : 0u);
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(b_ptr, live ? b_bytes : 0u);
    MOE_TILE_LOADS(a_rsrc, a_voff, A_LOADS, A);
    MOE_TILE_LOADS(b_rsrc, b_voff, B_LOADS, B);
    if (EPI == EPI_SWIGLU) {
      const __amdgpu_buffer_rsrc_t b2_rsrc = make_rsrc(b2_ptr, live ? b_bytes : 0u);
      MOE_TILE_LOADS(b2_rsrc, b_voff, B_LOADS, B + B_ROWS * ROW_BYTES);
    }
  };
#undef MOE_TILE_LOADS
  const int KT = K / KS;
  auto issue_prologue = [&]() {  // the first NST stages of the bound tile
    issue_stage(0, true, s0);
    issue_stage(1, 1 < KT, s1);
    if (NST == 4) {
      issue_stage(2, 2 < KT, s2);
      issue_stage(3, 3 < KT, s3);
    }
  };

  f32x16 acc[TB][FB];
  bf16x8 af[2][TB], wfr[2][FB];
  // The K loop of one tile, compiled once per number TBV of 32-row token blocks of this wavefront that
  // hold at least one valid row (a partial tile - an expert's last rows - multiplies only those blocks;
  // a wavefront with none still takes part in the loads and the barriers).
  constexpr int LOADS_PER_STAGE = A_LOADS + B_LOADS * (EPI == EPI_SWIGLU ? 2 : 1);
  constexpr int IN_FLIGHT = (NST - 2) * LOADS_PER_STAGE;  // loads allowed to be outstanding at the barrier
  static_assert(IN_FLIGHT < 64, "vmcnt is a 6-bit counter");
  // s_waitcnt immediate: vmcnt = IN_FLIGHT (bits 3:0 and 15:14), expcnt = 7 (no wait), lgkmcnt = 0
  constexpr int WAIT_IMM = (IN_FLIGHT & 15) | ((IN_FLIGHT >> 4) << 14) | (7 << 4);
  auto run_tile = [&](auto tbv_tag) {
    constexpr int TBV = decltype(tbv_tag)::value;
    constexpr int NFB = TBV > 0 ? FB : 0;  // weight fragments are needed only if there is a token block
    auto read_frags = [&](const unsigned char* A, const unsigned char* B, int ks, bf16x8 (&a)[TB], bf16x8 (&w)[FB]) {
#pragma unroll
      for (int i = 0; i < TBV; ++i) a[i] = *reinterpret_cast<const bf16x8*>(A + (a_base[i] ^ (ks << 5)));
#pragma unroll
      for (int j = 0; j < NFB; ++j) w[j] = *reinterpret_cast<const bf16x8*>(B + (w_base[j] ^ (ks << 5)));
    };
    auto mfma_all = [&](const bf16x8 (&a)[TB], const bf16x8 (&w)[FB]) {
#pragma unroll
      for (int i = 0; i < TBV; ++i)
#pragma unroll
        for (int j = 0; j < FB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[j], a[i], acc[i][j], 0, 0, 0);
    };
    // Asks the scheduler to alternate one MFMA with one LDS read, then the remaining MFMAs.
    auto interleave = [&]() {
      constexpr int READS = TBV + NFB, MFMAS = TBV * FB;
      constexpr int PAIRS = READS < MFMAS ? READS : MFMAS;
#pragma unroll
      for (int q = 0; q < PAIRS; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
      }
      if (MFMAS > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - PAIRS, 0);
    };
    // One K-step on the stage in `cur`.  On entry fr[0] holds the fragments of sub-step 0 of that stage
    // and the loads of the following NST-1 stages are in flight.  All sub-steps but the last multiply while
    // the next sub-step's fragments are read; then every wavefront waits until its own share of the NEXT
    // stage has landed (the younger NST-2 batches may stay in flight: loads retire in order) and until its
    // fragment reads are done, and the workgroup meets at one barrier; the current stage's buffer is then
    // refilled with stage kt+NST, and the last sub-step multiplies while sub-step 0 of the next stage is
    // read.
    auto step = [&](int kt, unsigned char* cur, unsigned char* nxt) {
#pragma unroll
      for (int ks = 0; ks + 1 < NSUB; ++ks) {
        read_frags(cur, cur + A_BYTES, ks + 1, af[(ks + 1) & 1], wfr[(ks + 1) & 1]);
        mfma_all(af[ks & 1], wfr[ks & 1]);
        interleave();
      }
      asm volatile("s_waitcnt %0\n\ts_barrier" ::"n"(WAIT_IMM) : "memory");
      issue_stage(kt + NST, kt + NST < KT, cur);
      read_frags(nxt, nxt + A_BYTES, 0, af[0], wfr[0]);
      mfma_all(af[(NSUB - 1) & 1], wfr[(NSUB - 1) & 1]);
      interleave();
    };
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
  };

  // ---- persistent loop over this workgroup's slots ------------------------------------------------
  TileInfo ti, nx;
  int nx_tok[GATHER ? A_LOADS : 1];
  bool have = walk.next(offsets, E, s_pref, ti);
  if (!have) return;
  if constexpr (GATHER) {
    fetch_rows(ti, nx_tok);
    gather_voff(nx_tok);
  }
  bind_tile(ti);
  issue_prologue();

  while (true) {
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Everything this wavefront has in flight (the tile's first stages; the previous tile's stores, which
    // do not retire in order with loads) completes, then the workgroup meets: stage 0 is readable.
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    // the next tile is known now; its gathered row indices travel while this tile is multiplied
    const bool have_nx = walk.next(offsets, E, s_pref, nx);
    if constexpr (GATHER) {
      if (have_nx) fetch_rows(nx, nx_tok);
    }
    // token blocks of this wavefront with at least one valid row (wave-uniform)
    const int tbv = min(TB, max(0, (ti.rows - wt * WTOK + 31) / 32));
    switch (tbv) {
      case 0: run_tile(std::integral_constant<int, 0>{}); break;
      case 1: run_tile(std::integral_constant<int, (1 < TB ? 1 : TB)>{}); break;
      case 2: run_tile(std::integral_constant<int, (2 < TB ? 2 : TB)>{}); break;
      case 3: run_tile(std::integral_constant<int, (3 < TB ? 3 : TB)>{}); break;
      case 4: run_tile(std::integral_constant<int, (4 < TB ? 4 : TB)>{}); break;
      default: run_tile(std::integral_constant<int, TB>{}); break;
    }

    // ---- next tile: bind it and request its first stages before this tile's epilogue ---------------
    const TileInfo done = ti;
    ti = nx;
    have = have_nx;
    if constexpr (GATHER) {
      if (have) gather_voff(nx_tok);
    }
    // every fragment read of real data finished before the last barrier; what the last sub-step read
    // afterwards is never used, so the stage buffers may be overwritten now
    if (have) {
      bind_tile(ti);
      issue_prologue();
    }

    // ---- epilogue: lane holds token (lane&31), features 8*i + 4*(lane>>5) + r of each 32x32 block ----
    const int feat0 = done.ntile * OUT_FEAT;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int trow = wt * WTOK + tb * 32 + frow;
      if (trow >= done.rows) continue;
      uint16_t* orow = out + (size_t)(done.row0 + trow) * N;
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
              const u32x2 b = *reinterpret_cast<const u32x2*>(bias + (size_t)done.expert * N + n);
              bv[0] = bf16_bits_to_f32(b.x & 0xffffu); bv[1] = bf16_bits_to_f32(b.x >> 16);
              bv[2] = bf16_bits_to_f32(b.y & 0xffffu); bv[3] = bf16_bits_to_f32(b.y >> 16);
            }
            uint32_t p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float u = acc[tb][fb][4 * i + r] + bv[r];
              if (EPI == EPI_GELU) u = gelu_table(u, s_phi);
              p[r] = f32_to_bf16_bits(u);
            }
            u32x2 v;
            v.x = p[0] | (p[1] << 16);
            v.y = p[2] | (p[3] << 16);
            *reinterpret_cast<u32x2*>(orow + n) = v;
          }
      }
    }
    if (!have) break;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // only zero-length loads and stores remain; retire them
#endif
}

template <int TOK, int FEAT, int WT, int WF, int KS, int NST, int WPE, int EPI>
int32_t launch(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb,
               const uint16_t* bias, const int32_t* offsets, uint16_t* out, const int32_t* row_map, int N, int K,
               hipStream_t s) {
  constexpr int OUT_FEAT = EPI == EPI_SWIGLU ? FEAT / 2 : FEAT;
  if (N % OUT_FEAT) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: N=%d is not a multiple of %d", N, OUT_FEAT);
  if (K % KS) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d is not a multiple of %d", K, KS);
  if ((int64_t)TOK * K * 2 >= ((int64_t)1 << 31)) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d too large", K);
  const int64_t rmax = max_rows(cfg);
  if (rmax == 0) return MOE_OK;
  int64_t mt = rmax / TOK + cfg->E;  // every expert may end in one partial tile
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS) {
    const int64_t by_cap = (int64_t)cfg->E * ((C + TOK - 1) / TOK);
    if (by_cap < mt) mt = by_cap;
  }
  const int64_t blocks = block_count(mt, N / OUT_FEAT);  // upper bound of the device's block count
  if (blocks > INT32_MAX / 64) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: too many tiles");
  // persistent: one workgroup per CU (the LDS stages leave room for one), a multiple of the XCD count;
  // fewer when even the upper bound of the tile count cannot occupy every CU
  const int64_t per_xcd = ((blocks + NUM_XCD - 1) / NUM_XCD) * CU_PER_XCD;  // tiles one XCD may own
  const int64_t grid = (per_xcd < CU_PER_XCD ? per_xcd : CU_PER_XCD) * NUM_XCD;
  // the gathering variant exists for the first GEMM's epilogues only
  auto kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, NST, WPE, EPI, false>;
  if constexpr (EPI != EPI_BIAS) {
    if (row_map) kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, NST, WPE, EPI, true>;
  } else {
    if (row_map) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: the second GEMM reads contiguous rows");
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WT * WF * 64), 0, s, act, wa, wb, bias, offsets, out, row_map,
                     cfg->T, cfg->E, N, K);
  return check_hip(hipGetLastError(), "grouped GEMM launch");
}

// MOESYS_GEMM_DEEP=1 selects four 32-deep LDS stages instead of two 64-deep ones.  Off by default:
// measured ~7 % slower on MI355X (twice the barriers, no gain from the longer prefetch distance).
bool deep_pipeline() {
  static const bool v = [] { const char* e = getenv("MOESYS_GEMM_DEEP"); return e && atoi(e) != 0; }();
  return v;
}

// Token-tile height.  256 rows is the default; 320 rows (10 MFMA row blocks, still within the 160 KB LDS)
// is chosen when, for the row count an evenly loaded expert would get, it saves enough whole rounds of
// NUM_CU tiles to pay for the taller tile (e.g. ~1024 rows per expert: 4 tiles of 320 instead of 5 of 256).
// The estimate only steers the choice; any routing is handled by either height.
int pick_tile_rows(const moe_config* cfg, int n_tiles) {
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

// One grouped GEMM.  256x256x64 tiles (8 wavefronts, the highest arithmetic intensity that fits the
// 160 KB LDS) whenever the feature count allows; feature counts that are multiples of 64 but not of 256
// use narrow tiles.
template <int EPI, int KSB, int NSB>
int32_t gemm_any(const moe_config* cfg, const uint16_t* a, const uint16_t* wa, const uint16_t* wb, const uint16_t* bias,
                 const int32_t* offsets, uint16_t* o, const int32_t* row_map, int N, int K, hipStream_t s) {
  constexpr int BF = EPI == EPI_SWIGLU ? 128 : 256;  // output features of the big tile
  if (N % BF == 0) {
    // (the 320-row tile has no registers to spare for the row gather)
    if (KSB == 64 && !row_map && pick_tile_rows(cfg, N / BF) == 320)
      return launch<320, 256, 2, 4, 64, 2, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, N, K, s);
    return launch<256, 256, 2, 4, KSB, NSB, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, N, K, s);
  }
  if constexpr (EPI == EPI_SWIGLU)
    return launch<128, 128, 2, 2, 64, 2, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, N, K, s);
  else
    return launch<128, 64, 4, 1, 64, 2, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, N, K, s);
}

}  // namespace

// row_map (nullable): row_to_assign; the token rows are then gathered from x[T, d_model] instead of read
// from a dispatched copy.
int32_t launch_gemm1_bf16(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                          void* h, const int32_t* row_map, hipStream_t s) {
  if (cfg->act == MOE_ACT_SWIGLU)
    return (deep_pipeline() ? gemm_any<EPI_SWIGLU, 32, 4> : gemm_any<EPI_SWIGLU, 64, 2>)(
        cfg, (const uint16_t*)xd, (const uint16_t*)w->w_gate_proj, (const uint16_t*)w->w_up, nullptr, offsets,
        (uint16_t*)h, row_map, cfg->d_ff, cfg->d_model, s);
  return (deep_pipeline() ? gemm_any<EPI_GELU, 32, 4> : gemm_any<EPI_GELU, 64, 2>)(
      cfg, (const uint16_t*)xd, (const uint16_t*)w->w1, nullptr, (const uint16_t*)w->b1, offsets, (uint16_t*)h, row_map,
      cfg->d_ff, cfg->d_model, s);
}

int32_t launch_gemm2_bf16(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                          void* yd, hipStream_t s) {
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  return (deep_pipeline() ? gemm_any<EPI_BIAS, 32, 4> : gemm_any<EPI_BIAS, 64, 2>)(
      cfg, (const uint16_t*)h, (const uint16_t*)(sw ? w->w_down : w->w2), nullptr,
      (const uint16_t*)(sw ? nullptr : w->b2), offsets, (uint16_t*)yd, nullptr, cfg->d_model, cfg->d_ff, s);
}

// The first GEMM can gather its rows from x when every byte offset into x fits the 32-bit buffer offset.
bool gemm1_can_gather(const moe_config* cfg) {
  return cfg->dtype == MOE_BF16 && (int64_t)cfg->T * cfg->d_model * 2 < ((int64_t)1 << 31);
}

}  // namespace moesys
