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
// CDNA4 mapping.  The kernel is persistent: one workgroup per CU; a workgroup's
// first tile is fixed, every further one is drawn from a per-XCD counter, so
// workgroups that drew short tiles draw more of them.  A workgroup owns a
// TOK x FEAT output tile and walks K in steps of KS = 64.  Operand tiles go from
// global memory straight into LDS (buffer_load ... lds, 16 bytes per lane, no
// register staging) as rows of KS bf16 whose 16-byte chunks are XOR-swizzled
// with the row index, so that the per-lane 16-byte fragment reads of
// v_mfma_f32_32x32x16_bf16 (32-row fragments) and v_mfma_f32_16x16x32_bf16
// (16-row fragments) are free of bank conflicts.  Two LDS stages rotate,
// with ONE barrier per K-step placed before the step's last sub-step, so that
// the first fragments of the next step are read under the tail of the current
// one.  A stage is requested in two halves, each spread between the MFMAs of
// one sub-step (a burst of loads would stall the issuing wavefronts, and with
// them the matrix pipes, while the texture path drains it), and one more load
// per K-step prefetches into L2 the lines that will be requested one K-step
// later (the operands stream from HBM; the stage loads themselves have less
// than one K-step to land).  The first stages of the NEXT tile, its bias and
// its gathered row indices are requested before the epilogue of the current
// one, so their latency hides under the activation and the stores.
// The MFMA "A" operand is the weight fragment and the "B" operand the
// activation fragment: the accumulator then holds, per lane, one token and runs
// of four consecutive output features, which store as packed 8-byte pieces.
// Rows past an expert's end are masked by the buffer descriptor (loads return
// zero, stores are skipped), never padded in memory.  Tiles are enumerated on
// the device from expert_offsets (no host round trip) in an order that makes
// the workgroups resident on one XCD share operand tiles in that XCD's L2, and
// the eight XCDs walk the same weight columns at the same time so that HBM
// serves each weight tile once.
//
// Clocks and power.  Under this kernel the MI355X draws its full board power
// and runs at 1.6-2.0 GHz, not at the 2.4 GHz its peak figure assumes (measured:
// shader clock counter against the 100 MHz reference counter, and the board's
// power sensor); in shader clocks the K loop keeps the matrix pipes ~80 % busy.
// At the power limit the rate follows the energy per flop, which is why the
// 16x16x32 instruction (half the accumulator registers moved per flop) is the
// one used wherever experts fill their tiles, see use_mi16().
#include <cstdlib>
#include <type_traits>
#include "moesys_internal.h"

// Optional phase timing, compiled in with -DMOESYS_GEMM_PROFILE (a separate library, never the product
// build): every wavefront sums the shader clocks it spends between its K-step barriers, waiting for its
// own loads, waiting at the barriers and in the epilogues, and reads the 100 MHz reference counter at both
// ends, which gives the shader clock frequency the kernel actually ran at.  moe_gemm_profile_set() points
// the kernels at a buffer of PROF_SLOTS uint64 per wavefront (first GEMM first, second GEMM behind it).
#ifdef MOESYS_GEMM_PROFILE
#define MOE_PROF(...) __VA_ARGS__
#else
#define MOE_PROF(...)
#endif

namespace moesys {
MOE_PROF(__device__ unsigned long long* g_gemm_prof = nullptr; constexpr int PROF_SLOTS = 16;)
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int NUM_XCD = 8;
constexpr int CU_PER_XCD = 32;
constexpr int NUM_CU = NUM_XCD * CU_PER_XCD;

// EPI_COMBINE: the second GEMM with the top-1 combine folded in: row r goes to token row_map[r] as
// residual + gate weight * (product + bias), rounded once.
// EPI_DGELU: the backward pass's recomputation of the first GEMM: out = aux * gelu'(product + bias), where aux
// [R, N] (passed as the residual; it may be out itself) is the gradient of the activations; the
// pre-activations never reach memory.
// EPI_DSWIGLU: the same for SwiGLU experts: the gate and up products g, u are recomputed on the SwiGLU tile and
// out [R, 2N] receives d_g = aux * u * silu'(g) in columns [0, N) and d_u = aux * silu(g) in columns [N, 2N).
enum Epi { EPI_GELU = 0, EPI_SWIGLU = 1, EPI_BIAS = 2, EPI_COMBINE = 3, EPI_DGELU = 4, EPI_DSWIGLU = 5 };
// tiles of a gate block and an up block side by side
constexpr bool swiglu_tile(int epi) { return epi == EPI_SWIGLU || epi == EPI_DSWIGLU; }

// Which MFMA multiplies.  Under these kernels the board sits at its power limit and the clock follows the energy
// an instruction stream costs; measured on MI355X with random bf16 operands in registers and nothing else going on,
// v_mfma_f32_16x16x32_bf16 delivers 2049 TFLOP/s and v_mfma_f32_32x32x16_bf16 1875 TFLOP/s at the same 1.3 kW (both
// 2.47 PFLOP/s on all-zero operands, at 755 W and 881 W).  The LDS traffic is the same for both: a wavefront's
// fragments per 32 values of the contraction index are (token rows + feature rows) x 64 bytes either way.  The
// 16x16x32 form is used where a wavefront's token blocks come in pairs (the loop alternates between them);
// bit e of the mask switches it on for epilogue e.
#ifndef MOE_MI16_MASK
#define MOE_MI16_MASK 0x3f
#endif
// The accumulators of one 32x32 block of the output: one 16-register MFMA result, or the four 4-register results of
// its 16x16 sub-blocks (number 2 * (token half) + (feature half)); element r of either is the same output element
// of the block's owner lane, see the epilogue.  (Separate types: a 16-register value cut into four operands makes
// the compiler copy registers around every MFMA once the accumulators live in the second half of the register file.)
template <bool MI16> struct AccBlock;
template <> struct AccBlock<false> {
  f32x16 v;
  __device__ __forceinline__ float get(int r) const { return v[r]; }
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] = 0.f;
  }
};
template <> struct AccBlock<true> {
  f32x4 q[4];
  __device__ __forceinline__ float get(int r) const { return q[r >> 2][r & 3]; }
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
};
// s_waitcnt operand: at most n vector memory operations in flight, no LDS or scalar one, exports untouched
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }
constexpr bool use_mi16(int tok, int wt, int epi) { return tok <= 256 && (tok / 32 / wt) % 2 == 0 && ((MOE_MI16_MASK >> epi) & 1); }

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// two floats -> two bf16 in one dword (lo in the low half): one v_cvt_pk_bf16_f32, round to nearest even
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// gelu(u) = u * Phi(u).  Phi comes from a table in LDS: PHI_N entries on x_i = -PHI_RANGE + i / PHI_SCALE, filled
// once per workgroup with the exact erf, and read with linear interpolation.  An entry is the line through
// (x_i, Phi(x_i)) and (x_i+1, Phi(x_i+1)) as (intercept, slope) in u itself, so that the interpolation is one
// fused multiply-add of u (no fractional part to extract; the intercept is of order one, its rounding 1e-7).
// Interpolation error <= h^2/8 * max|Phi''| = (1/64)^2 / 8 * 0.242 = 7.4e-6, far below the
// bf16 rounding of h; outside the range Phi is 0 or 1 to 6e-16.  A table read plus ~8 ALU operations
// replaces ~50 for the library erff: the activation runs on every element of h while the matrix pipes
// wait, so its instruction count is what the GEMM1 epilogue costs.
constexpr int PHI_N = 1024;
constexpr float PHI_RANGE = 8.0f, PHI_SCALE = 64.0f;

__device__ __forceinline__ void fill_phi_table(f32x2* tab) {
  for (int i = threadIdx.x; i < PHI_N; i += blockDim.x) {
    const float x0 = -PHI_RANGE + (float)i / PHI_SCALE, x1 = -PHI_RANGE + (float)(i + 1) / PHI_SCALE;
    const float p0 = 0.5f * erfcf(-x0 * 0.70710678118654752f), p1 = 0.5f * erfcf(-x1 * 0.70710678118654752f);
    // the two end cells also serve everything outside the range: constants there (Phi is 0 or 1 to 6e-16)
    const float slope = (i == 0 || i == PHI_N - 1) ? 0.f : (p1 - p0) * PHI_SCALE;
    tab[i] = f32x2{p0 - slope * x0, slope};
  }
}
// LDS address of the table cell of u (entries of 8 bytes).  u is clamped into the range, scaled to bytes and added
// to 2^23 + the table's own LDS address: at that magnitude a float's unit in the last place is 1, so the sum's
// low mantissa bits ARE the rounded address, and masking the low three bits (the table is 8-byte aligned) and the
// bits above the LDS leaves the cell's address.  (Rounding to nearest instead of down moves the upper sixteenth
// of a cell to the next cell's line, read h/16 outside its cell: error f'' h^2 / 32, below the h^2 / 8 inside a
// cell.)  Three instructions (clamp, multiply-add, mask) where convert-to-integer, shift and base add took four.
constexpr float PHI_CLAMP_HI = PHI_RANGE - 1.0f / 256.0f;
typedef __attribute__((address_space(3))) const f32x2* phi_lds_ptr;
// the addend of phi_cell(): 2^23 + (offset of u = 0 in bytes) + the table's LDS address
__device__ __forceinline__ float phi_addend(const f32x2* tab) {
  const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)tab;
  return 8388608.0f + PHI_RANGE * PHI_SCALE * 8.0f + (float)base;  // (all integers below 2^24: exact)
}
// The read is written as table base + (address - table base): the two constants cancel in the generated code, and
// the compiler still knows which LDS object is read.  With a bare integer address it cannot tell the read from
// the LDS writes of the direct-to-LDS loads in flight (the next tile's first stages) and waits for all of them.
__device__ __forceinline__ f32x2 phi_cell(float u, float addend, const f32x2* tab) {
  const float c = __builtin_amdgcn_fmed3f(u, -PHI_RANGE, PHI_CLAMP_HI);
  const float tm = fmaf(c, PHI_SCALE * 8.0f, addend);
  const uint32_t addr = __float_as_uint(tm) & 0x3fff8u;  // (LDS addresses are below 2^18)
  const auto base = (__attribute__((address_space(3))) const char*)tab;
  return *(phi_lds_ptr)(base + (addr - (uint32_t)(uintptr_t)base));
}
// B values at a time, in three passes: table positions, the B table reads back to back, the
// interpolations.  (One value at a time the compiler waits for every read before it starts the next
// value, and the epilogue then runs at the latency of the LDS instead of at the rate of the vector ALU.)
template <int B>
__device__ __forceinline__ void gelu_table_n(float* u, float addend, const f32x2* tab) {
  f32x2 e[B];
#pragma unroll
  for (int r = 0; r < B; ++r) e[r] = phi_cell(u[r], addend, tab);
#pragma unroll
  for (int r = 0; r < B; ++r) u[r] *= fmaf(u[r], e[r].y, e[r].x);
}
// The backward pass's table: gelu'(u) = Phi(u) + u phi(u) on the same grid, filled with the exact erf and exp.
// Interpolation error <= h^2/8 * max|third derivative of gelu| = (1/64)^2 / 8 * 0.8 = 2.5e-5 on a factor of
// order one, far below the bf16 rounding of the product; outside the range gelu' is 0 or 1 to 1e-13.
__device__ __forceinline__ float gelu_prime_exact(float x) {
  return 0.5f * erfcf(-x * 0.70710678118654752f) + x * 0.3989422804014327f * expf(-0.5f * x * x);
}
__device__ __forceinline__ void fill_gelu_prime_table(f32x2* tab) {
  for (int i = threadIdx.x; i < PHI_N; i += blockDim.x) {
    const float x0 = -PHI_RANGE + (float)i / PHI_SCALE;
    const float g0 = gelu_prime_exact(x0), g1 = gelu_prime_exact(-PHI_RANGE + (float)(i + 1) / PHI_SCALE);
    const float slope = (i == 0 || i == PHI_N - 1) ? 0.f : (g1 - g0) * PHI_SCALE;  // (end cells: constants)
    tab[i] = f32x2{g0 - slope * x0, slope};  // (intercept, slope), as in the forward table
  }
}
// u[r] <- dh[r] * gelu'(u[r]), gelu' read from its table like Phi in the forward pass
template <int B>
__device__ __forceinline__ void dgelu_table_n(float* u, const float* dh, float addend, const f32x2* tab) {
  f32x2 e[B];
#pragma unroll
  for (int r = 0; r < B; ++r) e[r] = phi_cell(u[r], addend, tab);
#pragma unroll
  for (int r = 0; r < B; ++r) u[r] = dh[r] * fmaf(u[r], e[r].y, e[r].x);
}
__device__ __forceinline__ float silu(float u) { return u * __builtin_amdgcn_rcpf(1.f + __expf(-u)); }

struct TileInfo {
  int expert, row0, rows;  // first dispatched row and valid rows (<= TOK) of this tile
  int ntile;               // feature tile index
  int pm, gm;              // this tile is number pm of the gm tiles of its block that use the same weight tile
  int pn, gn;              // ... and number pn of the gn that use the same token tile
};

// Tile order.  Token tiles (of all experts, in row order) are grouped GM at a time and feature tiles GN
// at a time, GM*GN <= 32 = the CUs of one XCD, so that an XCD's workgroups reuse GM activation tiles and
// GN weight tiles out of its L2.  Workgroup w (on XCD w mod 8: the hardware hands workgroups to XCDs round
// robin) works on blocks b = 8q + xcd of up to 32 tiles, which are laid out so that
// the eight XCDs work on eight token groups of the SAME feature group at the same time (one HBM read of
// those weights serves all of them through the shared cache level).  A trailing partial set of token
// groups is spread over the XCDs feature group by feature group instead, to keep them equally loaded.
#ifndef MOE_GROUP_N
#define MOE_GROUP_N 8
#endif
__host__ __device__ inline int group_n(int n_tiles) { return n_tiles < MOE_GROUP_N ? n_tiles : MOE_GROUP_N; }

// Token tiling of one expert with n rows, for a kernel whose tile holds up to `cap` rows: the fewest tiles
// that can hold them, ceil(n / cap), with the rows spread over them as evenly as whole units allow (a unit =
// one 32-row MFMA block per wavefront row, the granularity at which a tile's K loop gets cheaper).  E.g. 1049
// rows under cap 320: 17 units of 64 rows in 4 tiles of 5,4,4,4 units.
__host__ __device__ inline int token_tiles(int n, int cap) { return (n + cap - 1) / cap; }
// s_pref[e] = number of token tiles of experts < e ; s_pref[E] = total.  Whole workgroup.
__device__ __forceinline__ void count_token_tiles(const int32_t* __restrict__ offsets, int E, int cap, int* s_pref) {
  for (int e = threadIdx.x; e < E; e += blockDim.x) s_pref[e + 1] = token_tiles(offsets[e + 1] - offsets[e], cap);
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
// takes number j first and then whatever number the XCD's counter hands out next (`want` is set by the
// caller before each call and must grow): workgroups that drew short tiles simply draw more of them.
// floor(a / b) for 0 <= a, 1 <= b and a quotient below 2^22, without the forty-odd instructions of the general
// 32-bit division: a reciprocal estimate is within one of the quotient, the exact remainder corrects it.  (The walk
// below runs once per tile on every wavefront while the matrix pipes wait, and is mostly divisions.)
__device__ __forceinline__ int div_small(int a, int b) {
  int q = (int)((float)a * __builtin_amdgcn_rcpf((float)b));
  const int r = a - q * b;
  q += r >= b ? 1 : 0;
  q -= r < 0 ? 1 : 0;
  return q;
}
// the same for operands that every lane holds alike: the quotient goes back to a scalar register
__device__ __forceinline__ int div_small_uniform(int a, int b) { return __builtin_amdgcn_readfirstlane(div_small(a, b)); }

template <int TOK, int UNIT>
struct TileWalker {
  int MT, NT, GM, GN, MG, NG;
  int xcd, G;
  int b, msg, rem;  // this workgroup's current block b = NUM_XCD * q + xcd, and b = msg * NUM_XCD * NG + rem
  int base, want;

  __device__ __forceinline__ void init(int mt_total, int n_tiles) {
    MT = mt_total; NT = n_tiles;
    GN = group_n(n_tiles); GM = CU_PER_XCD / GN;
    MG = (MT + GM - 1) / GM; NG = (NT + GN - 1) / GN;
    xcd = blockIdx.x % NUM_XCD; G = gridDim.x / NUM_XCD;
    b = xcd; msg = 0; rem = xcd;  // (xcd < NUM_XCD <= NUM_XCD * NG)
    base = 0; want = blockIdx.x / NUM_XCD;
  }
  // Next tile of this workgroup; false when there is none.  All values are wave-uniform; the whole wavefront
  // calls it (the search for the expert is one read per lane and a ballot).
  __device__ __forceinline__ bool next(const int32_t* __restrict__ offsets, int E, const int* s_pref, TileInfo& ti) {
    const int n_blocks = MG * NG;
    while (true) {
      if (b >= n_blocks) return false;
      const int P = min(NUM_XCD, MG - msg * NUM_XCD);
      static_assert(NUM_XCD == 8, "the shifts below");
      const int ng = P == NUM_XCD ? rem >> 3 : div_small_uniform(rem, P);
      const int mg = msg * NUM_XCD + (rem - ng * P);
      const int gm = min(GM, MT - mg * GM), gn = min(GN, NT - ng * GN);
      const int cnt = gm * gn;
      if (want < base + cnt) {
        const int r = want - base;  // (below 32)
        const int rq = gn == 8 ? r >> 3 : div_small_uniform(r, gn);
        const int mt = mg * GM + rq, nt = ng * GN + (r - rq * gn);
        // largest e with s_pref[e] <= mt = the number of e in 1..E with s_pref[e] <= mt (s_pref does not
        // decrease, and s_pref[E] = MT > mt)
        const int lane = threadIdx.x & 63;
        int lo = 0;
        for (int e0 = 0; e0 < E; e0 += 64) {
          const int e = e0 + lane + 1;
          lo += __builtin_popcountll(__ballot(e <= E && s_pref[min(e, E)] <= mt));
        }
        // every lane computed the same values; say so to the compiler (they feed scalar descriptors)
        lo = __builtin_amdgcn_readfirstlane(lo);
        ti.expert = lo;
        // tile m of the expert's nt tiles: the units are dealt out evenly, the first `extra` tiles hold one more
        const int e0 = offsets[lo], n_rows = offsets[lo + 1] - e0;
        const int m = mt - s_pref[lo], nt_e = s_pref[lo + 1] - s_pref[lo];
        const int units = (n_rows + UNIT - 1) / UNIT, per = div_small_uniform(units, nt_e), extra = units - per * nt_e;
        const int u0 = m * per + min(m, extra), un = per + (m < extra ? 1 : 0);
        const int r0 = __builtin_amdgcn_readfirstlane(e0 + u0 * UNIT);
        ti.row0 = r0;
        ti.rows = __builtin_amdgcn_readfirstlane(min(un * UNIT, e0 + n_rows - r0));
        ti.ntile = __builtin_amdgcn_readfirstlane(nt);
        // who shares this tile's operands: the gn feature tiles of the block share the token tile; the weight
        // tile is shared by those of the block's token tiles that belong to the same expert
        const int m_lo = max(mg * GM, s_pref[lo]), m_hi = min(mg * GM + gm, s_pref[lo + 1]);
        ti.pm = __builtin_amdgcn_readfirstlane(mt - m_lo);
        ti.gm = __builtin_amdgcn_readfirstlane(m_hi - m_lo);
        ti.pn = __builtin_amdgcn_readfirstlane(r - rq * gn);
        ti.gn = __builtin_amdgcn_readfirstlane(gn);
        return true;
      }
      base += cnt;
      b += NUM_XCD;
      rem += NUM_XCD;
      if (rem >= NUM_XCD * NG) {
        rem -= NUM_XCD * NG;
        ++msg;
      }
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

// TOK x FEAT tile, WT x WF wavefronts, K-step KS, two LDS stages; each wavefront owns TOK/WT tokens (every
// WT-th 32-row block) x FEAT/WF LDS feature rows.  WPE = wavefronts per SIMD the register budget is sized for.
// HASB = false: the caller passed no bias; its staging and the two vector instructions per element that add it
// are compiled out (SwiGLU never has one).
template <int TOK, int FEAT, int WT, int WF, int KS, int WPE, int EPI, bool GATHER, bool HASB, bool MI16_>
__global__ __launch_bounds__(WT * WF * 64, WPE) void grouped_gemm_kernel(
    const uint16_t* __restrict__ act,     // [R, K]
    const uint16_t* __restrict__ wa,      // [E, N, K]   (W1 / Wg / W2)
    const uint16_t* __restrict__ wb,      // [E, N, K]   (Wu, SwiGLU only)
    const uint16_t* __restrict__ bias,    // [E, N] or NULL
    const int32_t* __restrict__ offsets,  // [E+1]
    uint16_t* out,                        // [R, N]; EPI_COMBINE: [T, N], may be the residual itself
    const int32_t* __restrict__ row_map,  // GATHER: row_to_assign; act is then x[T,K] and row r reads token row_map[r] mod T
                                          // EPI_COMBINE: row_to_assign with k = 1, i.e. the token of every row
    const float* __restrict__ gate_w,     // EPI_COMBINE: [T] gate weight of every token
    const uint16_t* residual,             // EPI_COMBINE: [T, N] or NULL
    const int64_t* __restrict__ eoff,     // [E] or NULL: expert e's weights (and bias) start eoff[e] elements after
                                          // wa/wb (bias) instead of e*N*K (e*N)
    int32_t* __restrict__ tile_ctr,       // [NUM_XCD] zero at launch: tiles handed out beyond each workgroup's first
    int32_t* __restrict__ clear_ctr,      // [NUM_XCD] or NULL: cleared here for the kernel that runs next
    int T, int E, int N, int K) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub (buffer descriptors are device-only types)
  constexpr int NW = WT * WF;
  constexpr int WFEAT = FEAT / WF;
  // 32x32 MFMA blocks per wavefront.  Token block i of wavefront row wt is block i*WT + wt of the tile: the
  // rows of a partly filled tile then spread evenly over the wavefront rows.
  constexpr int TB = TOK / 32 / WT, FB = WFEAT / 32;
  static_assert(TOK % (32 * WT) == 0, "tile/wavefront mismatch");
  constexpr int ROW_BYTES = KS * 2;               // one LDS row
  constexpr int CHUNKS = KS / 8;                  // 16-byte chunks per row
  constexpr int RPB = 256 / ROW_BYTES;            // rows per 256 bytes (the LDS bank period for 16-byte reads)
  constexpr int RPI = 1024 / ROW_BYTES;           // rows moved by one wave-wide 16-byte-per-lane load
  constexpr int NSUB = KS / 16;                   // MFMA sub-steps per K-step
  constexpr int A_BYTES = TOK * ROW_BYTES, B_BYTES = FEAT * ROW_BYTES;
  // SwiGLU: LDS feature rows [0,FEAT/2) come from Wg, [FEAT/2,FEAT) from Wu, for FEAT/2 output features
  constexpr int OUT_FEAT = swiglu_tile(EPI) ? FEAT / 2 : FEAT;
  constexpr int B_ROWS = OUT_FEAT;                                    // rows per weight matrix per tile
  constexpr int A_LOADS = TOK / RPI / NW, B_LOADS = B_ROWS / RPI / NW;  // wave-instructions per wavefront per stage
  static_assert(TOK % (RPI * NW) == 0 && B_ROWS % (RPI * NW) == 0, "tile/wavefront mismatch");
  // SwiGLU: a wavefront's FB blocks are FB/2 gate blocks followed by the FB/2 up blocks of the same features
  constexpr int FBH = swiglu_tile(EPI) ? FB / 2 : FB;
  static_assert(!swiglu_tile(EPI) || FB % 2 == 0, "SwiGLU wave tile is gate blocks + as many up blocks");
  static_assert(EPI != EPI_DSWIGLU || FB == 2, "the SwiGLU-gradient epilogue is written for one gate and one up block");
  static_assert(NSUB == 2 || NSUB == 4, "K-step is 32 or 64");  // (an even count: the fragment sets alternate)
  constexpr int ABUF = TOK > 256 ? 1 : 2;  // sets of token fragments, see `substep`
  constexpr bool MI16 = MI16_ && use_mi16(TOK, WT, EPI);  // 16x16x32 MFMAs, see `phase16`
  constexpr int PF_LEAD = 1;               // K-steps between a line's prefetch and the request of its stage (2 and 3
                                           // measured 1 % and 2 % slower at the large SwiGLU workload, none 4-8 %)
  constexpr int PF_MIN_KT = 64;            // shortest K loop (in K-steps) that prefetches, see bind_prefetch

  // LDS tile layout: row r keeps its logical 16-byte chunk c at physical chunk c ^ key(r), key(r) =
  // (r / RPB) mod CHUNKS.  The LDS serves 16 lanes x 16 B per clock over a 256-byte bank period; with this
  // key any 16 consecutive rows read at one logical chunk land on 16 distinct 16-byte bank groups
  // (measured conflict-free on gfx950, where keying on r mod 8 gives 2-way conflicts).
  // Two stages, each one array holding the token tile then the feature tile: separate arrays so
  // that the compiler can tell a stage being filled by LDS DMA from the stage being read.
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char s0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char s1[STAGE_BYTES];
  __shared__ f32x2 s_phi[EPI == EPI_GELU || EPI == EPI_DGELU ? PHI_N : 1];
  __shared__ int s_pref[MOE_MAX_EXPERTS + 1];
  __shared__ int s_next;  // number of this workgroup's next tile
  __shared__ int s_tok[GATHER ? NW * 64 : 1];  // assignment id of every row of the next tile
  static_assert(TOK <= NW * 64, "one thread per tile row");
  __shared__ __attribute__((aligned(256))) unsigned char s_sink[256];  // where prefetched dwords land (never read)
  // each wavefront's own slice of the tile's bias (WFEAT bf16 in the first bytes of its 256-byte slot); two
  // sets, because the next tile's bias is requested before the current tile's epilogue reads its own
  __shared__ __attribute__((aligned(256))) unsigned char s_bias[HASB ? 2 * NW * 256 : 256];
  // EPI_COMBINE: the token of every row of the tile, two sets like the bias
  __shared__ int s_rowtok[EPI == EPI_COMBINE ? 2 * NW * 64 : 1];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wt = wave / WF, wf = wave % WF;
  const uint32_t row_bytes = (uint32_t)K * 2u;
  const int n_tiles = N / OUT_FEAT;

  if (clear_ctr && blockIdx.x == 0 && tid < NUM_XCD) clear_ctr[tid] = 0;
  if (EPI == EPI_GELU) fill_phi_table(s_phi);
  if (EPI == EPI_DGELU) fill_gelu_prime_table(s_phi);
  const float phi_add = phi_addend(s_phi);
  count_token_tiles(offsets, E, TOK, s_pref);  // ends with a barrier: s_pref and the table are visible
  TileWalker<TOK, 32 * WT> walk;
  walk.init(s_pref[E], n_tiles);

  // ---- per-lane offsets of every direct-to-LDS load, LDS fragment addresses ----------------------
  // (with a row map the token-tile offsets are recomputed per tile from the gathered token indices)
  int a_voff[A_LOADS];
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
  // Row gather: the assignment ids of a tile's rows travel from row_map into s_tok (one dword per thread,
  // straight into LDS; threads past the tile's last row re-read its last entry), and once they have landed
  // and a barrier has passed, every lane turns the ids of its rows into offsets into x.
  auto fetch_rows = [&](const TileInfo& t) {
    const int32_t* src = row_map + t.row0 + min(tid, t.rows - 1);
    __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(s_tok + wave * 64), 4, 0, 0);
  };
  auto token_of = [&](int r) {
    int t = s_tok[r];
    while (t >= T) t -= T;  // assignment id j*T + t -> token (j < k <= 8)
    return t;
  };
  auto gather_voff = [&](const TileInfo& t) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      const int r = (i * NW + wave) * RPI + lane / CHUNKS;
      a_voff[i] = r < t.rows ? token_of(r) * (int)row_bytes + a_chunk(i) : 0x7fffffff;  // out of range: reads zero
    }
  };
  // Weight rows are never masked, so their row block can travel in the scalar offset: one per-lane offset
  // serves every load (the swizzle key of a lane's row is the same in every load, see the assert).
  static_assert((NW * (RPI / RPB)) % CHUNKS == 0, "a lane's swizzle key must not depend on the load index");
  const int b_voff = (lane / CHUNKS) * (int)row_bytes + a_chunk(0);
  const int b_blk = NW * RPI * (int)row_bytes;  // distance between the rows of consecutive loads
  // LDS byte address of this lane's fragment row with chunk key folded in: the chunk of K sub-step ks is
  // (2*ks + half) ^ key = (half ^ key) ^ 2*ks, i.e. base ^ (ks << 5).
  // (16x16x32: a fragment is 16 rows x 32 values, lane = row + 16 * chunk; sub-step kk of 32 values is chunks
  // 4*kk .. 4*kk+3, i.e. base ^ (kk << 6); a 32-row block is two such fragments 16 rows apart, same key)
  const int frow = MI16 ? lane & 15 : lane & 31, fhalf = MI16 ? lane >> 4 : lane >> 5;
  // Block i of this wavefront lies a whole number of 32-row blocks further on, which leaves the key alone:
  // one base per operand, the block goes into the constant part of the address.
  static_assert(32 % (RPB * CHUNKS) == 0, "the swizzle key must repeat every 32 rows");
  static_assert(!MI16 || (16 % (RPB * CHUNKS) == 0 && KS == 64), "16-row fragments: the key must repeat every 16 rows");
  const int a_row0 = wt * 32 + frow;
  const int w_row0 = (swiglu_tile(EPI) ? wf * (WFEAT / 2) : wf * WFEAT) + frow;  // SwiGLU: gate rows, the up rows FEAT/2 further
  const int a_base = a_row0 * ROW_BYTES + ((fhalf ^ ((a_row0 / RPB) % CHUNKS)) << 4);
  const int w_base = w_row0 * ROW_BYTES + ((fhalf ^ ((w_row0 / RPB) % CHUNKS)) << 4);
  constexpr int A_BLK = WT * 32 * ROW_BYTES;                                   // next token block of this wavefront
  // byte distance of feature block j from block 0 (SwiGLU: blocks FBH.. are the up rows of blocks 0..FBH-1)
  auto w_blk = [](int j) constexpr { return (swiglu_tile(EPI) ? (j / FBH) * (FEAT / 2) + (j % FBH) * 32 : j * 32) * ROW_BYTES; };

  // ---- the current tile's operand windows (wave-uniform) ----------------------------------------
  const uint16_t *a_ptr = act, *b_ptr = wa, *b2_ptr = wa;
  uint32_t a_bytes = 0;
  const uint32_t b_bytes = (uint32_t)B_ROWS * row_bytes;
  auto bind_tile = [&](const TileInfo& t) {
    const size_t woff = (eoff ? (size_t)eoff[t.expert] : (size_t)t.expert * N * K) + (size_t)t.ntile * OUT_FEAT * K;
    a_ptr = GATHER ? act : act + (size_t)t.row0 * K;
    b_ptr = wa + woff;
    b2_ptr = (swiglu_tile(EPI) ? wb : wa) + woff;
    a_bytes = (GATHER ? (uint32_t)T : (uint32_t)t.rows) * row_bytes;
  };
  // One instruction moves 64 lanes x 16 B = RPI rows of a tile; lane l lands at row l/CHUNKS, physical
  // chunk l%CHUNKS, and voff addresses the logical chunk that the swizzle maps there.  The K-step is
  // selected by the uniform offset.  `live` = false turns the loads into no-ops (zero-length descriptors),
  // so that the number of loads in flight at every wait is fixed.  A stage is requested in two halves
  // (token rows, then weight rows) at two different points of the K loop, see `step`.
  auto issue_tokens = [&](int kt, bool live, unsigned char* stage) {
    const int koff = kt * ROW_BYTES;
    const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(a_ptr, live ? a_bytes : 0u);
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (__attribute__((address_space(3))) void*)(stage + (i * NW + wave) * 1024), 16,
                                               a_voff[i], koff, 0, 0);
  };
  auto issue_weights = [&](int kt, bool live, unsigned char* stage) {
    unsigned char* B = stage + A_BYTES;
    const int koff = kt * ROW_BYTES;
    const __amdgpu_buffer_rsrc_t b_rsrc = make_rsrc(b_ptr, live ? b_bytes : 0u);
    const int woff = koff + wave * RPI * (int)row_bytes;
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (__attribute__((address_space(3))) void*)(B + (i * NW + wave) * 1024), 16,
                                               b_voff, woff + i * b_blk, 0, 0);
    if (swiglu_tile(EPI)) {
      const __amdgpu_buffer_rsrc_t b2_rsrc = make_rsrc(b2_ptr, live ? b_bytes : 0u);
#pragma unroll
      for (int i = 0; i < B_LOADS; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            b2_rsrc, (__attribute__((address_space(3))) void*)(B + B_ROWS * ROW_BYTES + (i * NW + wave) * 1024), 16, b_voff,
            woff + i * b_blk, 0, 0);
    }
  };
  const int KT = K / KS;

  // L2 prefetch.  One instruction per wavefront and K-step touches one dword of a 128-byte line per lane
  // (it lands in a sink in LDS that nobody reads) PF_LEAD K-steps before the stage holding the line is
  // requested: the operands stream from HBM, and a stage whose lines still have to come from there takes
  // ~1.5 us to land where one found in L2 takes ~1.0 us (measured).  The gn workgroups of a block that
  // share a token tile each take a 1/gn slice of its rows and the gm workgroups that share a weight tile
  // a 1/gm slice of its rows, so every line is asked for once per XCD (asking from every workgroup doubles
  // the L2 request traffic and gains nothing).  Lanes without a line re-touch the tile's first weight line.
  // Measured on MI355X, the prefetch pays only where the K loop is long and its operands are shared (second
  // GEMM of the large SwiGLU workload +3.5 %, of the GPT-style one +2 %); with K of 1024-2048 or with weight
  // tiles that no other workgroup reads (few rows per expert: the kernel is then bound by HBM, not by
  // latency) it costs 5-20 %, so short K loops do not prefetch and unshared tiles are left out.
  const uint16_t* pf_ptr = wa;  // this lane's line at K-step 0 of the bound tile
  auto bind_prefetch = [&](const TileInfo& t) {
    const int a_lo = div_small_uniform(t.pn * TOK, t.gn), a_n = t.gn > 1 ? div_small_uniform((t.pn + 1) * TOK, t.gn) - a_lo : 0;
    const int b_lo = div_small_uniform(t.pm * FEAT, t.gm), b_n = t.gm > 1 ? div_small_uniform((t.pm + 1) * FEAT, t.gm) - b_lo : 0;
    pf_ptr = b_ptr;
    if (KT < PF_MIN_KT) return;
    if (tid < a_n) {
      const int ar = a_lo + tid;
      if (ar < t.rows) {
        if constexpr (GATHER) {
          pf_ptr = act + (size_t)token_of(ar) * K;
        } else {
          pf_ptr = a_ptr + (size_t)ar * K;
        }
      }
    } else if (tid - a_n < b_n) {
      const int br = b_lo + tid - a_n;  // LDS feature row: SwiGLU keeps the second matrix in rows B_ROWS...
      pf_ptr = br < B_ROWS ? b_ptr + (size_t)br * K : b2_ptr + (size_t)(br - B_ROWS) * K;
    }
  };
  auto issue_prefetch = [&](int kt) {  // the lines of K-step kt (past the last K-step: the last one again)
    const uint16_t* p = pf_ptr + (size_t)min(kt, KT - 1) * KS;
    __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) void*)p,
                                     (__attribute__((address_space(3))) void*)s_sink, 4, 0, 0);
  };
  int bias_set = 0;  // the set the bound tile's bias goes to
  auto issue_prologue = [&](const TileInfo& t) {  // stage 0, the token half of stage 1, the first prefetches, the bias
    issue_tokens(0, true, s0);
    issue_weights(0, true, s0);
    issue_tokens(1, 1 < KT, s1);
#pragma unroll
    for (int j = 1; j <= PF_LEAD; ++j) issue_prefetch(j);
    if constexpr (HASB) {
      // this wavefront's WFEAT bias values: lanes 0..WFEAT/2-1 move one dword each, the others read out of
      // range, which stores zeros
      const uint16_t* brow = bias + (eoff ? (size_t)eoff[t.expert] : (size_t)t.expert * N) +
                             (size_t)t.ntile * OUT_FEAT + wf * WFEAT;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(make_rsrc(brow, (uint32_t)WFEAT * 2u),
                                               (__attribute__((address_space(3))) void*)(s_bias + (bias_set * NW + wave) * 256), 4, lane * 4, 0, 0, 0);
    }
    if constexpr (EPI == EPI_COMBINE) {  // one row id per thread, threads past the last row re-read it
      const int32_t* src = row_map + t.row0 + min(tid, t.rows - 1);
      __builtin_amdgcn_global_load_lds((__attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)(s_rowtok + (bias_set * NW + wave) * 64), 4, 0, 0);
    }
  };

  // Tiles beyond a workgroup's first come from its XCD's counter.  One thread draws a number when a tile
  // starts; the value is published to the workgroup two K-steps later (by then the atomic has long
  // returned, so nobody waits for it) and turned into the next tile two K-steps after that, early enough
  // for the next tile's gathered row indices to arrive under the rest of the K loop.
  TileInfo ti, nx;
  bool have_nx = false;
  int drawn = 0;
  auto draw_next = [&]() {
    if (tid == 0) drawn = __hip_atomic_fetch_add(tile_ctr + walk.xcd, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  auto publish_next = [&]() {
    if (tid == 0) s_next = walk.G + drawn;
  };
  auto resolve_next = [&]() {
    walk.want = s_next;
    have_nx = walk.next(offsets, E, s_pref, nx);
    if constexpr (GATHER) {
      if (have_nx) fetch_rows(nx);
    }
  };

  MOE_PROF(struct { unsigned long long comp, vm, bar, steps, epi, tiles, tbar, start, last, c0, r0, ewait, tail, pro, walk; } pf = {};
           pf.c0 = __builtin_readcyclecounter(); pf.r0 = __builtin_amdgcn_s_memrealtime();)
  // (16x16x32: acc[i][j] holds the four 16x16 sub-blocks of the 32x32 block, four registers each, number
  // 2 * (token half) + (feature half); the fragment sets hold half of the token blocks, 16 rows at a time)
  AccBlock<MI16> acc[TB][FB];
  bf16x8 af[ABUF][MI16 ? (TB / 2) * 2 : TB], wfr[2][MI16 ? FB * 2 : FB];
  // The K loop of one tile, compiled once per number TBV of 32-row token blocks of this wavefront that
  // hold at least one valid row (a partial tile - an expert's last rows - multiplies only those blocks;
  // a wavefront with none still takes part in the loads and the barriers).
  constexpr int W_LOADS = B_LOADS * (swiglu_tile(EPI) ? 2 : 1);
  auto run_tile = [&](auto tbv_tag) {
    constexpr int TBV = decltype(tbv_tag)::value;
    constexpr int NFB = TBV > 0 ? FB : 0;  // weight fragments are needed only if there is a token block
    // Fragment reads and one sub-step: multiply with the fragments at hand (set `c`) while those of sub-step
    // `ks` of the stage at (A, B) are read (into set `c ^ 1`).  Two schedules:
    //  - two sets of token fragments (ABUF == 2): all reads of the next sub-step pair off with the first
    //    MFMAs of this one; fastest, needs 4*TB more registers;
    //  - one set (ABUF == 1, the 320-row tile): a token fragment is used by FB consecutive MFMAs only and is
    //    reloaded for the next sub-step right after them (it is next needed a whole sub-step later); only
    //    the weight fragments, which every token block uses, are kept twice.
    // The scheduler is asked to keep that order and to issue one of the VM global loads of this sub-step
    // after each MFMA (group) while there are any.  Spreading the loads matters: the texture path accepts
    // one 1 KB load per 16 clocks and the issuing wavefront waits when its queue is full, so a burst of
    // loads ahead of the MFMAs leaves the matrix pipes idle while the burst drains.
    auto read_w = [&](const unsigned char* B, int ks, auto& w) {
#pragma unroll
      for (int j = 0; j < NFB; ++j) w[j] = *reinterpret_cast<const bf16x8*>(B + (w_base ^ (ks << 5)) + w_blk(j));
    };
    auto read_a = [&](const unsigned char* A, int ks, bf16x8& a, int i) {
      a = *reinterpret_cast<const bf16x8*>(A + (a_base ^ (ks << 5)) + i * A_BLK);
    };
    auto substep = [&](const unsigned char* A, const unsigned char* B, int ks, int c, auto vm_tag) {
      constexpr int VM = decltype(vm_tag)::value;
      constexpr int MFMAS = TBV * FB;
      if constexpr (MI16) {
        return;  // (this wavefront's K loop is `step16`)
      } else {
      read_w(B, ks, wfr[c ^ 1]);
      if constexpr (ABUF == 2) {
#pragma unroll
        for (int i = 0; i < TBV; ++i) read_a(A, ks, af[c ^ 1][i], i);
#pragma unroll
        for (int i = 0; i < TBV; ++i)
#pragma unroll
          for (int j = 0; j < FB; ++j)
            acc[i][j].v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[c][j], af[c][i], acc[i][j].v, 0, 0, 0);
#pragma unroll
        for (int q = 0; q < MFMAS; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                      // MFMA
          if (q < TBV + NFB) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
          if (q < VM) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);         // VMEM
        }
      } else {
#pragma unroll
        for (int i = 0; i < TBV; ++i) {
#pragma unroll
          for (int j = 0; j < FB; ++j)
            acc[i][j].v = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[c][j], af[0][i], acc[i][j].v, 0, 0, 0);
          read_a(A, ks, af[0][i], i);
        }
        if (NFB) __builtin_amdgcn_sched_group_barrier(0x100, NFB, 0);
#pragma unroll
        for (int i = 0; i < TBV; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, FB, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
          constexpr int PER = (VM + TBV - 1) / (TBV ? TBV : 1);
#pragma unroll
          for (int p = 0; p < PER; ++p)
            if (i * PER + p < VM) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // VMEM
        }
      }
      }
    };
    // One K-step on the stage in `cur`.  On entry af/wfr[0] hold the fragments of sub-step 0 of that stage,
    // stage kt+1 has its token half in flight, and `nxt` (read by nobody since the last barrier) is free for
    // its weight half, which sub-step 0 requests, followed by the prefetch.  All sub-steps but the last
    // multiply while the next sub-step's fragments are read; then every wavefront waits until its share of
    // stage kt+1 has landed (the prefetch, younger than those loads, stays in flight: loads retire in
    // order) and until its fragment reads are done, and the workgroup meets at one barrier.  After it `cur`
    // is free: the last sub-step requests the token half of stage kt+2 into it and multiplies while
    // sub-step 0 of stage kt+1 is read.
    auto step = [&](int kt, unsigned char* cur, unsigned char* nxt) {
      issue_weights(kt + 1, kt + 1 < KT, nxt);
      issue_prefetch(kt + 1 + PF_LEAD);
      substep(cur, cur + A_BYTES, 1, 0, std::integral_constant<int, W_LOADS + 1>{});
#pragma unroll
      for (int ks = 1; ks + 1 < NSUB; ++ks) substep(cur, cur + A_BYTES, ks + 1, ks & 1, std::integral_constant<int, 0>{});
      MOE_PROF(__builtin_amdgcn_s_waitcnt(0xc07f); const unsigned long long t_a = __builtin_readcyclecounter();)
      __builtin_amdgcn_s_waitcnt(0x0071);  // vmcnt(1), expcnt untouched, lgkmcnt(0)
      MOE_PROF(const unsigned long long t_b = __builtin_readcyclecounter();)
      __builtin_amdgcn_s_barrier();
      MOE_PROF(const unsigned long long t_c = __builtin_readcyclecounter(); pf.comp += t_a - pf.last; pf.vm += t_b - t_a;
               pf.bar += t_c - t_b; pf.last = t_c; ++pf.steps;)
      issue_tokens(kt + 2, kt + 2 < KT, cur);
      substep(nxt, nxt + A_BYTES, 0, (NSUB - 1) & 1, std::integral_constant<int, A_LOADS>{});
    };
    // ---- the same with 16x16x32 MFMAs ----
    // A stage (64 values of the contraction index) is four phases: (kk, th) = (phase / 2, phase % 2) multiplies
    // values 32*kk .. 32*kk+31 for the token blocks 2*th and 2*th+1 of this wavefront (those of them that hold
    // rows).  A phase needs the 2*FB weight fragments of kk (kept twice: set kk & 1) and the up to four token
    // fragments of (kk, th) (kept twice: set phase & 1), and reads the next phase's token fragments, plus the
    // next kk's weight fragments when it is the last phase of its kk, while it multiplies: 16 MFMAs of half
    // the length and 4 or 8 fragment reads, where the 32x32x16 loop has 8 MFMAs and 6 reads per sub-step.
    constexpr int HTB = TB / 2;
    auto read_w16 = [&](const unsigned char* B, int kk, bf16x8 (&w)[MI16 ? FB * 2 : FB]) {
      if constexpr (MI16) {
#pragma unroll
        for (int j = 0; j < NFB; ++j)
#pragma unroll
          for (int fh = 0; fh < 2; ++fh)
            w[2 * j + fh] = *reinterpret_cast<const bf16x8*>(B + (w_base ^ (kk << 6)) + w_blk(j) + fh * 16 * ROW_BYTES);
      }
    };
    // token blocks of half th that hold rows
    auto blocks_of = [](int th) constexpr { return TBV - HTB * th < 0 ? 0 : (TBV - HTB * th > HTB ? HTB : TBV - HTB * th); };
    auto read_a16 = [&](const unsigned char* A, int kk, int th, auto nb_tag, bf16x8 (&a)[MI16 ? HTB * 2 : TB]) {
      if constexpr (MI16) {
#pragma unroll
        for (int i = 0; i < decltype(nb_tag)::value; ++i)
#pragma unroll
          for (int sh = 0; sh < 2; ++sh)
            a[2 * i + sh] = *reinterpret_cast<const bf16x8*>(A + (a_base ^ (kk << 6)) + (th * HTB + i) * A_BLK + sh * 16 * ROW_BYTES);
      }
    };
    // phase PH of the stage whose fragments are at hand; the fragments of phase (PH + 1) % 4 are read from (A, B),
    // which is the same stage, or the next one for PH = 3
    auto phase16 = [&](const unsigned char* A, const unsigned char* B, auto ph_tag, auto vm_tag) {
      if constexpr (MI16) {
        constexpr int PH = decltype(ph_tag)::value, VM = decltype(vm_tag)::value;
        constexpr int KK = PH / 2, TH = PH % 2, NPH = (PH + 1) % 4, NKK = NPH / 2, NTH = NPH % 2;
        constexpr int NB = blocks_of(TH), NNB = blocks_of(NTH);
        constexpr int MFMAS = NB * 2 * FB * 2;
        constexpr int READS = NNB * 2 + (NKK != KK ? NFB * 2 : 0);
        if constexpr (NKK != KK) read_w16(B, NKK, wfr[NKK & 1]);
        read_a16(A, NKK, NTH, std::integral_constant<int, NNB>{}, af[NPH & 1]);
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
          for (int j = 0; j < FB; ++j)
#pragma unroll
            for (int sh = 0; sh < 2; ++sh)
#pragma unroll
              for (int fh = 0; fh < 2; ++fh) {
                f32x4& c = acc[TH * HTB + i][j].q[2 * sh + fh];
                c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[KK & 1][2 * j + fh], af[PH & 1][2 * i + sh], c, 0, 0, 0);
              }
        // two MFMAs, then a fragment read and a global load while there are any
        constexpr int SLOTS = MFMAS / 2;
#pragma unroll
        for (int q = 0; q < SLOTS; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                 // MFMA
          if (q < READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // DS read
          if (q < VM) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);     // VMEM
        }
      }
    };
    auto step16 = [&](int kt, unsigned char* cur, unsigned char* nxt) {
      issue_weights(kt + 1, kt + 1 < KT, nxt);
      issue_prefetch(kt + 1 + PF_LEAD);
      phase16(cur, cur + A_BYTES, std::integral_constant<int, 0>{}, std::integral_constant<int, W_LOADS + 1>{});
      phase16(cur, cur + A_BYTES, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{});
      phase16(cur, cur + A_BYTES, std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{});
      MOE_PROF(__builtin_amdgcn_s_waitcnt(0xc07f); const unsigned long long t_a = __builtin_readcyclecounter();)
      __builtin_amdgcn_s_waitcnt(0x0071);  // vmcnt(1), expcnt untouched, lgkmcnt(0)
      MOE_PROF(const unsigned long long t_b = __builtin_readcyclecounter();)
      __builtin_amdgcn_s_barrier();
      MOE_PROF(const unsigned long long t_c = __builtin_readcyclecounter(); pf.comp += t_a - pf.last; pf.vm += t_b - t_a;
               pf.bar += t_c - t_b; pf.last = t_c; ++pf.steps;)
      issue_tokens(kt + 2, kt + 2 < KT, cur);
      phase16(nxt, nxt + A_BYTES, std::integral_constant<int, 3>{}, std::integral_constant<int, A_LOADS>{});
    };
    if constexpr (MI16) {
      read_w16(s0 + A_BYTES, 0, wfr[0]);
      read_a16(s0, 0, 0, std::integral_constant<int, blocks_of(0)>{}, af[0]);
    } else {
      read_w(s0 + A_BYTES, 0, wfr[0]);
#pragma unroll
      for (int i = 0; i < TBV; ++i) read_a(s0, 0, af[0][i], i);
    }
    auto any_step = [&](int kt, unsigned char* cur, unsigned char* nxt) {
      if constexpr (MI16) step16(kt, cur, nxt);
      else step(kt, cur, nxt);
    };
    int kt = 0;
    for (; kt + 1 < KT; kt += 2) {
      any_step(kt, s0, s1);
      any_step(kt + 1, s1, s0);
      if (kt == 0) publish_next();
      if (kt == 2) {  // the two K-steps since publish_next() each passed a barrier
        MOE_PROF(const unsigned long long t_r = __builtin_readcyclecounter();)
        resolve_next();
        MOE_PROF(pf.walk += __builtin_readcyclecounter() - t_r;)
      }
    }
    if (kt < KT) any_step(kt, s0, s1);
  };

  // ---- persistent loop over this workgroup's slots ------------------------------------------------
  bool have = walk.next(offsets, E, s_pref, ti);
  if (!have) return;
  if constexpr (GATHER) {
    fetch_rows(ti);
    __builtin_amdgcn_s_waitcnt(0x0070);
    __syncthreads();
    gather_voff(ti);
  }
  bind_tile(ti);
  bind_prefetch(ti);
  issue_prologue(ti);

  // stores per wavefront in the epilogue of a tile without missing rows (its loads, if any, are not counted: a
  // lower bound of what is issued after the next tile's first requests is what the wait below needs)
  constexpr int EPI_STORES = TB * 2 * (EPI == EPI_SWIGLU ? FBH : EPI == EPI_DSWIGLU ? 2 : FB);
  bool stores_behind = false;
  while (true) {
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
      for (int j = 0; j < FB; ++j) acc[i][j].clear();

    // The tile's first stages and bias have landed, then the workgroup meets: stage 0 is readable.  Vector memory
    // operations leave the counter in the order they were issued, and the previous tile's epilogue came after the
    // requests for this tile's first stages: when that epilogue issued every one of its EPI_STORES stores (a
    // wavefront whose rows all exist), waiting until no more than those are in flight is enough, and the stores
    // complete under the first K-step (whose own wait covers them, being older than its loads).
    MOE_PROF(const unsigned long long t_w = __builtin_readcyclecounter();)
    if (stores_behind) __builtin_amdgcn_s_waitcnt(waitcnt_vm(EPI_STORES));
    else __builtin_amdgcn_s_waitcnt(0x0070);
    MOE_PROF({ const unsigned long long t = __builtin_readcyclecounter(); if (pf.tiles) { pf.epi += t - pf.last; pf.ewait += t - t_w; } pf.last = t; })
    __builtin_amdgcn_s_barrier();
    MOE_PROF({ const unsigned long long t = __builtin_readcyclecounter(); if (pf.tiles) pf.tbar += t - pf.last; else pf.start = t - pf.c0;
               pf.last = t; ++pf.tiles; })
    draw_next();
    // token blocks of this wavefront with at least one valid row (wave-uniform)
    const int tbv = min(TB, max(0, (ti.rows - wt * 32 + 32 * WT - 1) / (32 * WT)));
    switch (tbv) {
      case 0: run_tile(std::integral_constant<int, 0>{}); break;
      case 1: run_tile(std::integral_constant<int, (1 < TB ? 1 : TB)>{}); break;
      case 2: run_tile(std::integral_constant<int, (2 < TB ? 2 : TB)>{}); break;
      case 3: run_tile(std::integral_constant<int, (3 < TB ? 3 : TB)>{}); break;
      case 4: run_tile(std::integral_constant<int, (4 < TB ? 4 : TB)>{}); break;
      default: run_tile(std::integral_constant<int, TB>{}); break;
    }
    if (KT < 4) {  // too few K-steps for the K loop to have done it
      if (KT < 2) publish_next();
      __syncthreads();
      resolve_next();
    }
    if (GATHER && KT < 6) {  // no K-step with its barrier has followed the request of the next tile's row ids
      __builtin_amdgcn_s_waitcnt(0x0070);
      __syncthreads();
    }

    // ---- next tile: bind it and request its first stages before this tile's epilogue ---------------
    MOE_PROF(const unsigned long long t_k = __builtin_readcyclecounter(); pf.tail += t_k - pf.last;)
    const TileInfo done = ti;
    ti = nx;
    have = have_nx;
    // every fragment read of real data finished before the last barrier; what the last sub-step read
    // afterwards is never used, so the stage buffers may be overwritten now
    const int done_set = bias_set;
    if (have) {
      bias_set ^= 1;
      if constexpr (GATHER) gather_voff(ti);
      bind_tile(ti);
      bind_prefetch(ti);
      issue_prologue(ti);
    }
    MOE_PROF(pf.pro += __builtin_readcyclecounter() - t_k;)
    __builtin_amdgcn_sched_barrier(0);  // the epilogue's stores stay behind those requests (the next tile's wait counts on it)

    // ---- epilogue: lane holds token (lane&31), features 8*i + 4*(lane>>5) + r of each 32x32 block ----
    // Lanes l and l+32 hold the two halves of the same token's 8-feature groups.  For a pair of groups
    // (i, i+1) they trade halves (v_permlane32_swap: the upper lanes' first operand against the lower lanes'
    // second), after which lane l owns all 8 features of group i and lane l+32 those of group i+1: one
    // 16-byte store per lane and pair instead of two 8-byte ones.
    // With 16x16x32 MFMAs a lane holds token (lane&15) of each 16-token half of the block and features
    // 4*(lane>>4) + r of each 16-feature half: registers 4*(2*sh + fh) + r of acc[tb][fb].  The code below is the
    // same for both with the pair index i0 = 0, 2 read as the token half sh = i0/2 and the member g of a pair
    // as the feature half: lanes l and l+16 hold features 4m..4m+3 and 4m+4..4m+7 of both feature halves and
    // trade (v_permlane16_swap), after which the even 16-lane row owns 8 features of the first half and the odd
    // row 8 of the second.
    const int feat0 = done.ntile * OUT_FEAT;
    // where this lane's four features of member g of pair i0 start inside a 32-feature block (before the trade)
    auto run_off = [&](int i0, int g) { return MI16 ? 16 * g + 4 * fhalf : 8 * (i0 + g) + 4 * fhalf; };
    // where the eight features this lane stores for pair i0 start (after the trade)
    auto store_off = [&](int i0) { return MI16 ? 16 * (fhalf & 1) + 8 * (fhalf >> 1) : 8 * (i0 + fhalf); };
    // this lane's row of the tile for token block tb and pair i0
    auto tile_row = [&](int tb, int i0) { return (tb * WT + wt) * 32 + (MI16 ? 16 * (i0 >> 1) : 0) + frow; };
    auto trade = [&](uint32_t x, uint32_t y) {
      if constexpr (MI16) return __builtin_amdgcn_permlane16_swap(x, y, false, false);
      else return __builtin_amdgcn_permlane32_swap(x, y, false, false);
    };
    auto store_pair = [&](uint16_t* orow, int n0, int i0, const float (&p)[8], bool live) {
      const u32x2 sx = trade(pack_bf16(p[0], p[1]), pack_bf16(p[4], p[5]));
      const u32x2 sy = trade(pack_bf16(p[2], p[3]), pack_bf16(p[6], p[7]));
      if (live) *reinterpret_cast<u32x4*>(orow + n0 + store_off(i0)) = u32x4{sx.x, sy.x, sx.y, sy.y};
    };
    constexpr int RSETS = MI16 ? 2 : 1;  // rows of a lane per token block
    int row_tok[TB * RSETS];   // EPI_COMBINE: token and gate weight of this lane's rows in every token block
    float row_gw[TB * RSETS];
    if constexpr (EPI == EPI_COMBINE) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int rs = 0; rs < RSETS; ++rs) {
          row_tok[tb * RSETS + rs] = s_rowtok[done_set * NW * 64 + min(tile_row(tb, 2 * rs), done.rows - 1)];
          row_gw[tb * RSETS + rs] = gate_w[row_tok[tb * RSETS + rs]];
        }
    }
    // EPI_DGELU: the activations' gradient for one (token block, feature block, group pair) step, loaded one
    // step ahead of its use in the layout of the stores: 16 bytes per lane, the 8 features this lane stores
    // (rows past the tile's last re-read the last row)
    auto aux_load = [&](int tb, int fb, int i0) {
      const int trow = min(tile_row(tb, i0), done.rows - 1);
      return *reinterpret_cast<const u32x4*>(residual + (size_t)(done.row0 + trow) * N + feat0 +
                                             (swiglu_tile(EPI) ? wf * 32 : wf * WFEAT + fb * 32) + store_off(i0));
    };
    u32x4 aux_next = {0u, 0u, 0u, 0u};
    if constexpr (EPI == EPI_DGELU || EPI == EPI_DSWIGLU) aux_next = aux_load(0, 0, 0);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      // 32x32x16: lanes l and l+32 share the row, they stay or leave together; the rows grow with tb, so nothing
      // after a skipped block is processed either.  16x16x32: a block is left when it holds no row at all (the
      // same for the whole wavefront); inside a block only the stores depend on the row, because the second
      // half's rows may lie past the end when the first half's do not.
      if (MI16 ? (tb * WT + wt) * 32 >= done.rows : tile_row(tb, 0) >= done.rows) continue;
      auto live_row = [&](int i0) { return !MI16 || tile_row(tb, i0) < done.rows; };
      auto out_row = [&](int i0) {
        return EPI == EPI_COMBINE ? (size_t)row_tok[tb * RSETS + (MI16 ? i0 >> 1 : 0)] : (size_t)(done.row0 + tile_row(tb, i0));
      };
      if constexpr (EPI == EPI_DSWIGLU) {
#pragma unroll
        for (int i0 = 0; i0 < 4; i0 += 2) {
          uint16_t* orow2 = out + out_row(i0) * (size_t)(2 * N);  // [d_g | d_u] rows
          // aux in the layout of the stores, the halves traded back (as in EPI_DGELU)
          const u32x2 sx = trade(aux_next.x, aux_next.z);
          const u32x2 sy = trade(aux_next.y, aux_next.w);
          if (i0 + 2 < 4) aux_next = aux_load(tb, 0, i0 + 2);
          else if (tb + 1 < TB) aux_next = aux_load(tb + 1, 0, 0);
          float pg[8], pu[8];
#pragma unroll
          for (int g = 0; g < 2; ++g) {
            const uint32_t lo = g ? sx.y : sx.x, hi = g ? sy.y : sy.x;
            const float dh[4] = {bf16_bits_to_f32(lo & 0xffffu), __uint_as_float(lo & 0xffff0000u),
                                 bf16_bits_to_f32(hi & 0xffffu), __uint_as_float(hi & 0xffff0000u)};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float gv = acc[tb][0].get(4 * (i0 + g) + q), uv = acc[tb][1].get(4 * (i0 + g) + q);
              const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-gv));   // sigmoid(g)
              const float ds = dh[q] * sg;
              pu[4 * g + q] = ds * gv;                                     // d_u = d_h * silu(g)
              pg[4 * g + q] = ds * uv * fmaf(gv, 1.f - sg, 1.f);           // d_g = d_h * u * s (1 + g (1 - s))
            }
          }
          store_pair(orow2, feat0 + wf * 32, i0, pg, live_row(i0));
          store_pair(orow2 + N, feat0 + wf * 32, i0, pu, live_row(i0));
        }
      } else if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int fb = 0; fb < FBH; ++fb)
#pragma unroll
          for (int i0 = 0; i0 < 4; i0 += 2) {
            float p[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) p[r] = silu(acc[tb][fb].get(4 * i0 + r)) * acc[tb][FBH + fb].get(4 * i0 + r);
            store_pair(out + out_row(i0) * N, feat0 + wf * (WFEAT / 2) + fb * 32, i0, p, live_row(i0));
          }
      } else {
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
          for (int i0 = 0; i0 < 4; i0 += 2) {
            const size_t orow_idx = out_row(i0);
            float p[8];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
              if constexpr (HASB) {
                // the bias sits in this wavefront's LDS slot since the tile's prologue
                const u32x2 b = *reinterpret_cast<const u32x2*>(s_bias + (done_set * NW + wave) * 256 +
                                                                (fb * 32 + run_off(i0, g)) * 2);
                p[4 * g + 0] = acc[tb][fb].get(4 * (i0 + g) + 0) + bf16_bits_to_f32(b.x & 0xffffu);
                p[4 * g + 1] = acc[tb][fb].get(4 * (i0 + g) + 1) + __uint_as_float(b.x & 0xffff0000u);
                p[4 * g + 2] = acc[tb][fb].get(4 * (i0 + g) + 2) + bf16_bits_to_f32(b.y & 0xffffu);
                p[4 * g + 3] = acc[tb][fb].get(4 * (i0 + g) + 3) + __uint_as_float(b.y & 0xffff0000u);
              } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) p[4 * g + q] = acc[tb][fb].get(4 * (i0 + g) + q);
              }
            }
            if (EPI == EPI_GELU) {
              constexpr int GB = TOK > 256 ? 4 : 8;  // (8 at a time in the 320-row kernel: at the register limit, no faster)
#pragma unroll
              for (int r = 0; r < 8; r += GB) gelu_table_n<GB>(p + r, phi_add, s_phi);
            }
            if constexpr (EPI == EPI_DGELU) {
              // (every element is read by the lane that multiplies it, before the lanes trade halves and before
              // that row segment is stored, so aux may be the output itself)
              float dh[8];
              // the store's trade of halves, backwards: every lane gets its own four features of both members
              // of the pair (element g of sx, sy: this lane's features of member g)
              const u32x2 sx = trade(aux_next.x, aux_next.z);
              const u32x2 sy = trade(aux_next.y, aux_next.w);
              {
                int ni0 = i0 + 2, nfb = fb, ntb = tb;
                if (ni0 == 4) { ni0 = 0; if (++nfb == FB) { nfb = 0; ++ntb; } }
                if (ntb < TB) aux_next = aux_load(ntb, nfb, ni0);
              }
#pragma unroll
              for (int g = 0; g < 2; ++g) {
                const u32x2 rv = {g ? sx.y : sx.x, g ? sy.y : sy.x};
                dh[4 * g + 0] = bf16_bits_to_f32(rv.x & 0xffffu);
                dh[4 * g + 1] = __uint_as_float(rv.x & 0xffff0000u);
                dh[4 * g + 2] = bf16_bits_to_f32(rv.y & 0xffffu);
                dh[4 * g + 3] = __uint_as_float(rv.y & 0xffff0000u);
              }
#pragma unroll
              for (int r = 0; r < 8; r += 4) dgelu_table_n<4>(p + r, dh + r, phi_add, s_phi);
            }
            if constexpr (EPI == EPI_COMBINE) {
              // before the lanes trade halves: this lane's 4 + 4 features of the residual row
              const float gw = row_gw[tb * RSETS + (MI16 ? i0 >> 1 : 0)];
#pragma unroll
              for (int g = 0; g < 2; ++g) {
                u32x2 rv = {0u, 0u};
                if (residual)
                  rv = *reinterpret_cast<const u32x2*>(residual + orow_idx * N + feat0 + wf * WFEAT + fb * 32 + run_off(i0, g));
                p[4 * g + 0] = __builtin_fmaf(gw, p[4 * g + 0], bf16_bits_to_f32(rv.x & 0xffffu));
                p[4 * g + 1] = __builtin_fmaf(gw, p[4 * g + 1], __uint_as_float(rv.x & 0xffff0000u));
                p[4 * g + 2] = __builtin_fmaf(gw, p[4 * g + 2], bf16_bits_to_f32(rv.y & 0xffffu));
                p[4 * g + 3] = __builtin_fmaf(gw, p[4 * g + 3], __uint_as_float(rv.y & 0xffff0000u));
              }
            }
            store_pair(out + orow_idx * N, feat0 + wf * WFEAT + fb * 32, i0, p, live_row(i0));
          }
      }
    }
    if (!have) break;
    // the epilogue above ran all its stores with every lane alive: this wavefront's last row of the tile exists
    stores_behind = done.rows >= ((TB - 1) * WT + wt + 1) * 32;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // only zero-length loads and stores remain; retire them
  MOE_PROF(if (g_gemm_prof && lane == 0) {
    unsigned long long* o = g_gemm_prof + ((size_t)(EPI >= EPI_BIAS ? NUM_CU : 0) * 8 + (size_t)blockIdx.x * NW + wave) * PROF_SLOTS;
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
    o[0] = pf.comp; o[1] = pf.vm; o[2] = pf.bar; o[3] = pf.steps; o[4] = pf.epi; o[5] = pf.tiles; o[6] = c1 - pf.last;
    o[7] = pf.tbar; o[8] = pf.start; o[9] = c1 - pf.c0; o[10] = pf.r0; o[11] = r1; o[12] = pf.ewait; o[13] = pf.tail; o[14] = pf.pro; o[15] = pf.walk;
  })
#endif
}

template <int TOK, int FEAT, int WT, int WF, int KS, int WPE, int EPI, bool MI16_ = false>
int32_t launch(const moe_config* cfg, const uint16_t* act, const uint16_t* wa, const uint16_t* wb,
               const uint16_t* bias, const int32_t* offsets, uint16_t* out, const int32_t* row_map,
               int32_t* tile_ctr, int32_t* clear_ctr, int N, int K, hipStream_t s, const int64_t* eoff,
               const float* gate_w = nullptr, const uint16_t* residual = nullptr) {
  constexpr int OUT_FEAT = swiglu_tile(EPI) ? FEAT / 2 : FEAT;
  if (N % OUT_FEAT) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: N=%d is not a multiple of %d", N, OUT_FEAT);
  if (K % KS) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d is not a multiple of %d", K, KS);
  if ((int64_t)TOK * K * 2 >= ((int64_t)1 << 31)) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: K=%d too large", K);
  const int64_t rmax = max_rows(cfg);
  if (rmax == 0) return MOE_OK;
  int64_t mt = rmax / TOK + cfg->E;  // every expert may end in one partial tile
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS) {
    const int64_t by_cap = (int64_t)cfg->E * token_tiles((int)(C > INT32_MAX - TOK ? INT32_MAX - TOK : C), TOK);
    if (by_cap < mt) mt = by_cap;
  }
  const int64_t blocks = block_count(mt, N / OUT_FEAT);  // upper bound of the device's block count
  if (blocks > INT32_MAX / 64) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: too many tiles");
  // persistent: one workgroup per CU (the LDS stages leave room for one), a multiple of the XCD count;
  // fewer when even the upper bound of the tile count cannot occupy every CU
  const int64_t per_xcd = ((blocks + NUM_XCD - 1) / NUM_XCD) * CU_PER_XCD;  // tiles one XCD may own
  const int64_t grid = (per_xcd < CU_PER_XCD ? per_xcd : CU_PER_XCD) * NUM_XCD;
  // the gathering variant exists for the first GEMM's epilogues only
  auto kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, WPE, EPI, false, false, MI16_>;
  if constexpr (EPI == EPI_DSWIGLU) {
    if (row_map || !residual || bias) return fail(MOE_ERR_INVALID_ARG, "grouped GEMM: the SwiGLU-gradient epilogue reads contiguous rows, needs the activations' gradient and has no bias");
  } else if constexpr (EPI == EPI_SWIGLU) {
    if (row_map) kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, WPE, EPI, true, false, MI16_>;
  } else {
    if (bias) kern = grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, WPE, EPI, false, true, MI16_>;
  }
  if constexpr (EPI == EPI_GELU) {
    if (row_map)
      kern = bias ? grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, WPE, EPI, true, true, MI16_>
                  : grouped_gemm_kernel<TOK, FEAT, WT, WF, KS, WPE, EPI, true, false, MI16_>;
  } else if constexpr (swiglu_tile(EPI)) {
  } else if constexpr (EPI == EPI_BIAS) {
    if (row_map) return fail(MOE_ERR_UNSUPPORTED, "grouped GEMM: the second GEMM reads contiguous rows");
  } else if constexpr (EPI == EPI_DGELU) {
    if (row_map || !residual) return fail(MOE_ERR_INVALID_ARG, "grouped GEMM: the activation-gradient epilogue reads contiguous rows and needs the activations' gradient");
  } else {
    if (!row_map || !gate_w || cfg->k != 1) return fail(MOE_ERR_INVALID_ARG, "grouped GEMM: combine epilogue needs k = 1, row map and gate weights");
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WT * WF * 64), 0, s, act, wa, wb, bias, offsets, out, row_map,
                     gate_w, residual, eoff, tile_ctr, clear_ctr, cfg->T, cfg->E, N, K);
  return check_hip(hipGetLastError(), "grouped GEMM launch");
}

// Tile capacity.  The 256-row kernel keeps two sets of token fragments and has the faster K loop; the
// 320-row kernel (10 MFMA row blocks, one set of token fragments, still within 160 KB of LDS and 256
// registers) needs fewer tiles when the rows of an expert do not fill whole 256-row tiles: e.g. ~1050 rows
// are 4 tiles of 4-5 units (of 64 rows) under capacity 320 and 5 tiles of 3-4 units under 256, and a tile's
// K loop does not get cheaper below ~4 units (with little to multiply it runs at the latency of its weight
// loads).  With few tiles what counts is whole rounds of NUM_CU: 16 such experts x 4 feature tiles are 256
// tiles (one round) or 320 (two).  The choice is made for the row count an evenly loaded expert would get,
// with head-room for uneven routing and capped by the capacity; either kernel handles any routing.
int pick_tile_rows(const moe_config* cfg, int n_tiles) {
  const int forced = tuning(MOE_TUNE_GEMM_TILE_ROWS);
  if (forced == 256 || forced == 320) return forced;
  const int64_t A = (int64_t)cfg->k * cfg->T;
  int64_t rows = (A + cfg->E - 1) / cfg->E;
  rows += (rows * 2 + 24) / 25;  // 8 % head-room
  const int64_t C = moe_capacity(cfg);
  if (rows > C) rows = C;
  if (rows < 1) rows = 1;
  if (rows > (1 << 24)) return 256;
  int best = 256;
  double best_cost = -1;
  for (int cap : {256, 320}) {
    const int n = token_tiles((int)rows, cap);
    const double units = (double)((rows + 63) / 64) / n;       // per tile
    const double per_tile = (cap > 256 ? 1.05 : 1.0) * (units < 4.0 ? 4.0 : units);
    const double tiles = (double)cfg->E * n * n_tiles;
    // up to two rounds every workgroup's time is that of the largest tiles; beyond, the drawn tiles even out
    const bool few = tiles <= 2 * NUM_CU;
    const double rounds = few ? (double)((int64_t)(tiles + NUM_CU - 1) / NUM_CU) : tiles / NUM_CU;
    const double cost = rounds * (few ? (cap > 256 ? 1.05 : 1.0) * (double)(int64_t)(units + 0.999) : per_tile);
    if (best_cost < 0 || cost < best_cost) { best = cap; best_cost = cost; }
  }
  return best;
}

// The 16x16x32 loop is used where an evenly loaded expert fills whole tiles; with few rows per expert (the kernel is
// then bound by streaming the weights, and half of the loop's phases have nothing to multiply) the 32x32x16 loop
// measured 3 % faster.
bool prefer_mi16(const moe_config* cfg) {
  const int forced = tuning(MOE_TUNE_GEMM_MFMA);
  if (forced) return forced == 16;
  int64_t rows = ((int64_t)cfg->k * cfg->T + cfg->E - 1) / cfg->E;
  const int64_t C = moe_capacity(cfg);
  if (C != MOE_DROPLESS && rows > C) rows = C;
  return rows >= 192;
}

// One grouped GEMM.  256x256x64 tiles (8 wavefronts, the highest arithmetic intensity that fits the
// 160 KB LDS) whenever the feature count allows; feature counts that are multiples of 64 but not of 256
// use narrow tiles.
template <int EPI>
int32_t gemm_any(const moe_config* cfg, const uint16_t* a, const uint16_t* wa, const uint16_t* wb, const uint16_t* bias,
                 const int32_t* offsets, uint16_t* o, const int32_t* row_map, int32_t* tile_ctr, int32_t* clear_ctr, int N,
                 int K, hipStream_t s, const int64_t* eoff, const float* gate_w = nullptr,
                 const uint16_t* residual = nullptr) {
  constexpr int BF = swiglu_tile(EPI) ? 128 : 256;  // output features of the big tile
  if (N % BF == 0) {
    if (pick_tile_rows(cfg, N / BF) == 320)
      return launch<320, 256, 2, 4, 64, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, tile_ctr, clear_ctr, N, K, s, eoff, gate_w, residual);
    if (use_mi16(256, 2, EPI) && prefer_mi16(cfg))
      return launch<256, 256, 2, 4, 64, 2, EPI, true>(cfg, a, wa, wb, bias, offsets, o, row_map, tile_ctr, clear_ctr, N, K, s, eoff, gate_w, residual);
    return launch<256, 256, 2, 4, 64, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, tile_ctr, clear_ctr, N, K, s, eoff, gate_w, residual);
  }
  if constexpr (swiglu_tile(EPI))
    return launch<128, 128, 2, 2, 64, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, tile_ctr, clear_ctr, N, K, s, eoff, gate_w, residual);
  else
    return launch<128, 64, 4, 1, 64, 2, EPI>(cfg, a, wa, wb, bias, offsets, o, row_map, tile_ctr, clear_ctr, N, K, s, eoff, gate_w, residual);
}

}  // namespace

// steps of very few tokens (no expert has more than a handful of rows) take the matrix-vector kernels
bool expert_gemv_applies(const moe_config* cfg, int N, int K);
int32_t launch_expert_gemv_bf16(int epi, const moe_config* cfg, const void* act, const void* wa, const void* wb, const void* bias,
                                const int32_t* offsets, void* out, const int32_t* row_map, const float* gate_w,
                                const void* residual, const int64_t* eoff, int N, int K, hipStream_t s);

// row_map (nullable): row_to_assign; the token rows are then gathered from x[T, d_model] instead of read
// from a dispatched copy.
int32_t launch_gemm1_bf16(const moe_config* cfg, const moe_weights* w, const void* xd, const int32_t* offsets,
                          void* h, const int32_t* row_map, int32_t* tile_counters, hipStream_t s) {
  if (expert_gemv_applies(cfg, cfg->d_ff, cfg->d_model)) {
    if (cfg->act == MOE_ACT_SWIGLU)
      return launch_expert_gemv_bf16(EPI_SWIGLU, cfg, xd, w->w_gate_proj, w->w_up, nullptr, offsets, h, row_map, nullptr, nullptr,
                                     w->expert_elem_offset, cfg->d_ff, cfg->d_model, s);
    return launch_expert_gemv_bf16(EPI_GELU, cfg, xd, w->w1, nullptr, w->b1, offsets, h, row_map, nullptr, nullptr,
                                   w->expert_elem_offset, cfg->d_ff, cfg->d_model, s);
  }
  // the first GEMM draws from counters [0,8) and clears [8,16) for the second, which in turn clears [0,8): after
  // the pair has run the first GEMM's counters are back at zero, so the expert half of a layer can run again
  // on the same routing tables
  if (cfg->act == MOE_ACT_SWIGLU)
    return gemm_any<EPI_SWIGLU>(
        cfg, (const uint16_t*)xd, (const uint16_t*)w->w_gate_proj, (const uint16_t*)w->w_up, nullptr, offsets,
        (uint16_t*)h, row_map, tile_counters, tile_counters + NUM_XCD, cfg->d_ff, cfg->d_model, s, w->expert_elem_offset);
  return gemm_any<EPI_GELU>(
      cfg, (const uint16_t*)xd, (const uint16_t*)w->w1, nullptr, (const uint16_t*)w->b1, offsets, (uint16_t*)h, row_map,
      tile_counters, tile_counters + NUM_XCD, cfg->d_ff, cfg->d_model, s, w->expert_elem_offset);
}

int32_t launch_gemm2_bf16(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                          void* yd, int32_t* tile_counters, hipStream_t s) {
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  if (expert_gemv_applies(cfg, cfg->d_model, cfg->d_ff))
    return launch_expert_gemv_bf16(EPI_BIAS, cfg, h, sw ? w->w_down : w->w2, nullptr, sw ? nullptr : w->b2, offsets, yd, nullptr,
                                   nullptr, nullptr, w->expert_elem_offset, cfg->d_model, cfg->d_ff, s);
  return gemm_any<EPI_BIAS>(
      cfg, (const uint16_t*)h, (const uint16_t*)(sw ? w->w_down : w->w2), nullptr,
      (const uint16_t*)(sw ? nullptr : w->b2), offsets, (uint16_t*)yd, nullptr, tile_counters + NUM_XCD, tile_counters,
      cfg->d_model, cfg->d_ff, s, w->expert_elem_offset);
}

// The second GEMM with the top-1 combine in its epilogue: out[T, d_model] rows of the tokens that kept their
// expert are written here, the others by the caller.
int32_t launch_gemm2_combine_bf16(const moe_config* cfg, const moe_weights* w, const void* h, const int32_t* offsets,
                                  const int32_t* row_to_assign, const float* topk_w, const void* residual, void* out,
                                  int32_t* tile_counters, hipStream_t s) {
  const bool sw = cfg->act == MOE_ACT_SWIGLU;
  if (expert_gemv_applies(cfg, cfg->d_model, cfg->d_ff))
    return launch_expert_gemv_bf16(EPI_COMBINE, cfg, h, sw ? w->w_down : w->w2, nullptr, sw ? nullptr : w->b2, offsets, out,
                                   row_to_assign, topk_w, residual, w->expert_elem_offset, cfg->d_model, cfg->d_ff, s);
  return gemm_any<EPI_COMBINE>(
      cfg, (const uint16_t*)h, (const uint16_t*)(sw ? w->w_down : w->w2), nullptr,
      (const uint16_t*)(sw ? nullptr : w->b2), offsets, (uint16_t*)out, row_to_assign, tile_counters + NUM_XCD, tile_counters,
      cfg->d_model, cfg->d_ff, s, w->expert_elem_offset, topk_w, (const uint16_t*)residual);
}

// A plain grouped product out[r, n] = sum_k act[r, k] * w_e[n, k] (+ bias_e[n]) with the second GEMM's kernel:
// what the backward pass needs for its input gradients (on the weights' transposed copies) and for
// recomputing the pre-activations.  counters8: eight zeroed ints.
int32_t launch_grouped_matmul_bf16(const moe_config* cfg, const void* act, const void* w, const void* bias,
                                   const int32_t* offsets, void* out, int N, int K, int32_t* counters8, hipStream_t s) {
  return gemm_any<EPI_BIAS>(cfg, (const uint16_t*)act, (const uint16_t*)w, nullptr, (const uint16_t*)bias, offsets,
                            (uint16_t*)out, nullptr, counters8, nullptr, N, K, s, nullptr);
}

// d_u[r, n] = d_h[r, n] * gelu'(sum_k xd[r, k] * w1_e[n, k] + b1_e[n]): the first GEMM recomputed for the backward
// pass with the activation's derivative in its epilogue.  d_u may be d_h.  counters8: eight zeroed ints.
int32_t launch_gemm1_dgelu_bf16(const moe_config* cfg, const void* xd, const void* w1, const void* b1,
                                const int32_t* offsets, const void* d_h, void* d_u, int32_t* counters8, hipStream_t s) {
  return gemm_any<EPI_DGELU>(cfg, (const uint16_t*)xd, (const uint16_t*)w1, nullptr, (const uint16_t*)b1, offsets,
                             (uint16_t*)d_u, nullptr, counters8, nullptr, cfg->d_ff, cfg->d_model, s, nullptr, nullptr,
                             (const uint16_t*)d_h);
}

// SwiGLU experts: dgu[r, 0:N] = d_h * u * silu'(g), dgu[r, N:2N] = d_h * silu(g) with g = xd Wg_e^T, u = xd Wu_e^T
// recomputed (N = d_ff; dgu [R, 2N]).  counters8: eight zeroed ints.
int32_t launch_gemm1_dswiglu_bf16(const moe_config* cfg, const void* xd, const void* w_gate, const void* w_up,
                                  const int32_t* offsets, const void* d_h, void* dgu, int32_t* counters8, hipStream_t s) {
  return gemm_any<EPI_DSWIGLU>(cfg, (const uint16_t*)xd, (const uint16_t*)w_gate, (const uint16_t*)w_up, nullptr, offsets,
                               (uint16_t*)dgu, nullptr, counters8, nullptr, cfg->d_ff, cfg->d_model, s, nullptr, nullptr,
                               (const uint16_t*)d_h);
}

// The first GEMM can gather its rows from x when every byte offset into x fits the 32-bit buffer offset.
bool gemm1_can_gather(const moe_config* cfg) {
  return cfg->dtype == MOE_BF16 && (int64_t)cfg->T * cfg->d_model * 2 < ((int64_t)1 << 31);
}

}  // namespace moesys

#ifdef MOESYS_GEMM_PROFILE
// buf: device, 2 * 256 * 8 * 16 uint64, zeroed by the caller; NULL switches the recording off.
extern "C" int32_t moe_gemm_profile_set(unsigned long long* buf) {
  return moesys::check_hip(hipMemcpyToSymbol(HIP_SYMBOL(moesys::g_gemm_prof), &buf, sizeof(buf)), "hipMemcpyToSymbol");
}
#endif
