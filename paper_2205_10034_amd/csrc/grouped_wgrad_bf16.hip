// Grouped weight-gradient GEMM of the expert FFN's backward pass:
//
//   C_e[n1, n2] = sum over the rows r of expert e of A[r, n1] * B[r, n2]        (fp32 output)
//
// e.g. dW2_e = d_y_e^T h_e and dW1_e = d_u_e^T xd_e for OUTPUT_MAJOR weights.  The paper's system is a
// training system (Section 3.2) but gives no kernel; this is the chain rule on the expert FFN of the
// forward pass.  The contraction runs over an expert's rows, the SLOW index of both row-major operands,
// and its length differs per expert.
//
// CDNA4 mapping.  One workgroup (8 wavefronts, 2 x 4) per 256 x 256 tile of one expert's C; it walks the
// expert's rows 32 at a time.  Both operand chunks [32 rows x 256 columns] go from global memory straight
// into LDS as they are (buffer_load ... lds, 16 bytes per lane; rows past the expert's end read as zero
// through the buffer descriptor, so the ragged length needs no padding), three stages deep.  The MFMA
// operand fragments need 8 consecutive contraction indices per lane, i.e. a COLUMN of the LDS tile: they
// are read with gfx950's transposing LDS read (ds_read_b64_tr_b16: within 16 lanes, lane i supplies a
// chunk of four 16-bit values M[i][0..3] and lane L receives M[(L mod 16)/4 + 4j][L mod 4]); with lane i
// supplying row r0 + i/4, column chunk i mod 4, lane L receives rows r0..r0+3 of column n0 + L mod 16, so
// two reads make one fragment.  The 16-byte slot index of a row is XORed with 4*(row mod 4), which lets
// the two 16-lane groups of a 32-lane pass hit all 64 banks once.
// The first MFMA operand is the n2 side, so that a lane ends up with runs of four consecutive n2 of one
// n1: 16-byte fp32 stores.
// Tile order.  The 8 XCDs have an L2 each, and the hardware deals workgroups out to them round robin.  A tile
// streams a 256-column slab of A and one of B; tiles of one expert with the same n1 (n2) tile share the A (B)
// slab.  Workgroups are therefore numbered so that the 32 that start together on one XCD are a block of
// BY x BX tiles of ONE expert (BX = min(8, n2 tiles), BY = 32 / BX): BY + BX slabs for 32 tiles through that L2
// instead of the 6 for 8 that the plain (n2, n1, expert) grid order gives at 16 x 4 tiles per expert.
// Column sums of A per expert (the bias gradients: db2_e = sum_r d_y[r, :], db1_e = sum_r d_u[r, :]) come from
// the same fragments: the workgroups of the first n2 tile multiply one n1 fragment per wavefront and K-step
// by a fragment of ones (one more MFMA on top of eight), which leaves the column's sum in every element of
// that accumulator.  No extra pass over A.
#include "moesys_internal.h"

namespace moesys {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int WG_N = 256;        // tile edge (both n1 and n2)
constexpr int WG_KS = 32;        // rows per K-step
constexpr int WG_ROW = WG_N * 2; // bytes of one LDS row
constexpr int WG_CHUNK = WG_KS * WG_ROW;  // one operand chunk: 16 KB
constexpr int WG_STAGES = 3;
constexpr int WG_WAVES = 8;
constexpr int WG_LOADS = WG_CHUNK / 1024 / WG_WAVES;  // wave-wide 1 KB loads per wavefront, operand and stage: 2

#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t wg_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
#endif

template <bool COLSUM, bool OUT_BF16>
__global__ __launch_bounds__(WG_WAVES * 64, 2) void grouped_wgrad_kernel(
    const uint16_t* __restrict__ a,       // [R, N1]
    const uint16_t* __restrict__ b,       // [R, N2]
    const int32_t* __restrict__ offsets,  // [E+1]
    void* __restrict__ c_out,             // [E, N1, N2] float32, or bfloat16 (OUT_BF16: one rounding of the fp32 sums)
    float* __restrict__ a_colsum,         // COLSUM: [E, N1]
    int N1, int N2, int E, int BY, int BX) {
#if defined(__HIP_DEVICE_COMPILE__)
  // one array per stage: the compiler can then tell the stage being filled from the one being read
  __shared__ __attribute__((aligned(1024))) unsigned char s0[2 * WG_CHUNK];
  __shared__ __attribute__((aligned(1024))) unsigned char s1[2 * WG_CHUNK];
  __shared__ __attribute__((aligned(1024))) unsigned char s2[2 * WG_CHUNK];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int w1 = wave >> 2, w2 = wave & 3;  // this wavefront: n1 columns [128*w1, +128), n2 columns [64*w2, +64)
  // workgroup -> (expert, n1 tile, n2 tile): see "Tile order" above
  const int n1t = N1 / WG_N, n2t = N2 / WG_N;
  const int nby = (n1t + BY - 1) / BY, nbx = (n2t + BX - 1) / BX;
  const int slot = blockIdx.x / 8;                            // position in this XCD's sequence of workgroups
  const int blk = (slot / (BY * BX)) * 8 + (int)(blockIdx.x % 8);  // blocks are dealt out to the XCDs in turn
  const int in_blk = slot % (BY * BX);
  const int e = blk / (nby * nbx);
  const int ty = ((blk / nbx) % nby) * BY + in_blk / BX, tx = (blk % nbx) * BX + in_blk % BX;
  if (e >= E || ty >= n1t || tx >= n2t) return;                // (wave-uniform: padding of the grid and of partial blocks)
  const int row0 = offsets[e], rows = offsets[e + 1] - row0;
  const int t1 = ty * WG_N, t2 = tx * WG_N;
  const size_t c_tile = ((size_t)e * N1 + t1) * N2 + t2;  // element offset of this tile in c
  const int KT = (rows + WG_KS - 1) / WG_KS;

  // ---- direct-to-LDS loads: one instruction = 2 rows of a chunk; lane -> (row = lane / 32, physical slot =
  // lane % 32), which holds the logical slot (lane % 32) ^ key(row), key = 4 * (row mod 4).  Wavefront w
  // moves rows 2w, 2w+1 and 16 + 2w, 16 + 2w + 1.
  const int ld_row = 2 * wave + (lane >> 5);
  const int ld_slot = (lane & 31) ^ (4 * (ld_row & 3));
  const uint32_t a_pitch = (uint32_t)N1 * 2u, b_pitch = (uint32_t)N2 * 2u;
  const int a_voff = ld_row * (int)a_pitch + (t1 * 2 + ld_slot * 16);
  const int b_voff = ld_row * (int)b_pitch + (t2 * 2 + ld_slot * 16);
  const uint16_t* a_base = a + (size_t)row0 * N1;
  const uint16_t* b_base = b + (size_t)row0 * N2;
  const uint32_t a_bytes = (uint32_t)rows * a_pitch, b_bytes = (uint32_t)rows * b_pitch;
  auto issue = [&](int kt, unsigned char* stage) {
    const bool live = kt < KT;
    const __amdgpu_buffer_rsrc_t ra = wg_rsrc(a_base, live ? a_bytes : 0u), rb = wg_rsrc(b_base, live ? b_bytes : 0u);
    const int r0 = kt * WG_KS;
#pragma unroll
    for (int i = 0; i < WG_LOADS; ++i) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void*)(stage + (i * WG_WAVES + wave) * 1024), 16,
                                               a_voff, (r0 + 16 * i) * (int)a_pitch, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (__attribute__((address_space(3))) void*)(stage + WG_CHUNK + (i * WG_WAVES + wave) * 1024), 16,
                                               b_voff, (r0 + 16 * i) * (int)b_pitch, 0, 0);
    }
  };

  // ---- transposing fragment reads: lane L, 16-lane group g = L / 16, i = L mod 16 supplies row
  // 8*(g/2) + 4*h + i/4 (h = 0, 1: the two halves of its 8 contraction indices), columns 16*(g%2) + 4*(i%4)..+3
  // of the 32-column block; key(row) = 4 * ((i/4) mod 4) for every row it supplies.
  const int g = lane >> 4, li = lane & 15;
  const int fr_row = 8 * (g >> 1) + (li >> 2);                 // + 4*h + 16*ks
  const int fr_col = 16 * (g & 1) + 4 * (li & 3);              // column inside the 32-column block
  const int fr_key = 4 * ((li >> 2) & 3);
  auto frag_addr = [&](int col0) {  // byte offset of this lane's chunk for the block starting at column col0, row part excluded
    const int col = col0 + fr_col;
    return (((col >> 3) ^ fr_key) << 4) + ((col >> 2) & 1) * 8;
  };
  int n1_addr[4], n2_addr[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) n1_addr[i] = frag_addr(128 * w1 + 32 * i) + fr_row * WG_ROW;
#pragma unroll
  for (int j = 0; j < 2; ++j) n2_addr[j] = frag_addr(64 * w2 + 32 * j) + fr_row * WG_ROW;
  auto read_frag = [&](const unsigned char* chunk, int addr, int ks) {
    const unsigned char* p = chunk + addr + ks * 16 * WG_ROW;
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p);
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p + 4 * WG_ROW));
    bf16x8 f;
    const bf16x4 l4 = __builtin_bit_cast(bf16x4, lo), h4 = __builtin_bit_cast(bf16x4, hi);
#pragma unroll
    for (int q = 0; q < 4; ++q) { f[q] = l4[q]; f[4 + q] = h4[q]; }
    return f;
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // column sums: wavefront (w1, w2) of the first n2 tile's workgroups sums the n1 block i = w2 of its 128 columns
  const bool do_colsum = COLSUM && tx == 0;
  f32x16 acc_sum;
  bf16x8 ones;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_sum[v] = 0.f;
#pragma unroll
  for (int v = 0; v < 8; ++v) ones[v] = (__bf16)1.0f;

  auto compute = [&](const unsigned char* stage) {
#pragma unroll
    for (int ks = 0; ks < WG_KS / 16; ++ks) {
      bf16x8 f1[4], f2[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) f1[i] = read_frag(stage, n1_addr[i], ks);
#pragma unroll
      for (int j = 0; j < 2; ++j) f2[j] = read_frag(stage + WG_CHUNK, n2_addr[j], ks);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[j], f1[i], acc[i][j], 0, 0, 0);
      if constexpr (COLSUM) {
        if (do_colsum) {
          const bf16x8 mine = w2 == 0 ? f1[0] : w2 == 1 ? f1[1] : w2 == 2 ? f1[2] : f1[3];
          acc_sum = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, mine, acc_sum, 0, 0, 0);
        }
      }
    }
  };

  // ---- K loop, three stages: the loads of K-steps kt+1 and kt+2 stay in flight while K-step kt is
  // multiplied (past the last K-step the loads are zero-length, so the count in flight is the same)
  issue(0, s0);
  issue(1, s1);
  issue(2, s2);
  constexpr int PER_STAGE = 2 * WG_LOADS;  // loads per wavefront and stage
  static_assert(PER_STAGE == 4, "the wait below leaves two stages (8 loads) in flight");
  for (int kt = 0; kt < KT; kt += 3) {
    __builtin_amdgcn_s_waitcnt(0x0f78);  // vmcnt(8) only: this wavefront's share of the stage has landed
    __builtin_amdgcn_s_barrier();
    compute(s0);
    __builtin_amdgcn_s_barrier();
    issue(kt + 3, s0);
    if (kt + 1 < KT) {
      __builtin_amdgcn_s_waitcnt(0x0f78);
      __builtin_amdgcn_s_barrier();
      compute(s1);
      __builtin_amdgcn_s_barrier();
    }
    issue(kt + 4, s1);
    if (kt + 2 < KT) {
      __builtin_amdgcn_s_waitcnt(0x0f78);
      __builtin_amdgcn_s_barrier();
      compute(s2);
      __builtin_amdgcn_s_barrier();
    }
    issue(kt + 5, s2);
  }
  __builtin_amdgcn_s_waitcnt(0x0070);  // the zero-length tail loads retire

  // ---- epilogue: lane holds n1 = lane & 31 of each n1 block and n2 = 8*q + 4*(lane >> 5) + 0..3 of each n2 block
  const int o1 = lane & 31, o2 = 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const size_t crow = c_tile + (size_t)(128 * w1 + 32 * i + o1) * N2 + 64 * w2;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if constexpr (OUT_BF16) {
        // lanes l and l + 32 hold columns 8q + 0..3 and 8q + 4..7 of the same row: for a pair (q, q + 1) they trade
        // halves, after which lane l stores the eight columns of q and lane l + 32 those of q + 1 (16 bytes each;
        // 8-byte stores of half as many bytes took as long as the float32 ones)
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
          auto pk = [&](int qq, int r) {
            const bf16x2 h = __builtin_convertvector(f32x2{acc[i][j][4 * qq + r], acc[i][j][4 * qq + r + 1]}, bf16x2);
            return __builtin_bit_cast(uint32_t, h);
          };
          const u32x2 sx = __builtin_amdgcn_permlane32_swap(pk(q, 0), pk(q + 1, 0), false, false);
          const u32x2 sy = __builtin_amdgcn_permlane32_swap(pk(q, 2), pk(q + 1, 2), false, false);
          *reinterpret_cast<u32x4*>((uint16_t*)c_out + crow + 32 * j + 8 * (q + (lane >> 5))) = u32x4{sx.x, sy.x, sx.y, sy.y};
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = {acc[i][j][4 * q + 0], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4*>((float*)c_out + crow + o2 + 32 * j + 8 * q) = v;
        }
      }
    }
  }
  if constexpr (COLSUM) {
    // every element of acc_sum in lane l (and l + 32) is the sum of column 128*w1 + 32*w2 + (l & 31)
    if (do_colsum && lane < 32) a_colsum[(size_t)e * N1 + t1 + 128 * w1 + 32 * w2 + lane] = acc_sum[0];
  }
#endif
}

}  // namespace

int32_t launch_wgrad_bf16(const uint16_t* a, const uint16_t* b, const int32_t* offsets, void* c, int c_dtype, float* a_colsum, int E,
                          int N1, int N2, int64_t max_rows_per_expert, hipStream_t s) {
  if (c_dtype != MOE_F32 && c_dtype != MOE_BF16) return fail(MOE_ERR_INVALID_ARG, "weight gradient: output type must be MOE_F32 or MOE_BF16");
  if (N1 % WG_N || N2 % WG_N) return fail(MOE_ERR_UNSUPPORTED, "weight gradient: N1=%d and N2=%d must be multiples of %d", N1, N2, WG_N);
  const int64_t widest = N1 > N2 ? N1 : N2;
  if ((max_rows_per_expert + WG_KS) * widest * 2 >= ((int64_t)1 << 31))
    return fail(MOE_ERR_UNSUPPORTED, "weight gradient: an expert's operand block exceeds 2 GiB");
  const int n1t = N1 / WG_N, n2t = N2 / WG_N;
  const int BX = n2t < 8 ? n2t : 8, BY = 32 / BX;  // (BX in 1..8, so BY * BX is 32, or 28, 30 for BX = 7, 5, 6, 3)
  const int64_t blocks = (int64_t)E * ((n1t + BY - 1) / BY) * ((n2t + BX - 1) / BX);
  const int64_t wgs = ((blocks + 7) / 8) * 8 * BY * BX;
  if (wgs > INT32_MAX) return fail(MOE_ERR_UNSUPPORTED, "weight gradient: too many tiles");
  const dim3 grid((unsigned)wgs), block(WG_WAVES * 64);
  const bool h = c_dtype == MOE_BF16;
  auto kern = a_colsum ? (h ? grouped_wgrad_kernel<true, true> : grouped_wgrad_kernel<true, false>)
                       : (h ? grouped_wgrad_kernel<false, true> : grouped_wgrad_kernel<false, false>);
  hipLaunchKernelGGL(kern, grid, block, 0, s, a, b, offsets, c, a_colsum, N1, N2, E, BY, BX);
  return check_hip(hipGetLastError(), "weight gradient launch");
}

}  // namespace moesys

using namespace moesys;

extern "C" int32_t moe_expert_wgrad(const void* a, const void* b, const int32_t* expert_offsets, void* c, int32_t c_dtype,
                                    float* a_column_sums, int32_t E, int32_t N1, int32_t N2, int64_t max_rows_per_expert,
                                    void* stream) {
  if (!a || !b || !expert_offsets || !c) return fail(MOE_ERR_INVALID_ARG, "moe_expert_wgrad: NULL argument");
  if (E < 1 || E > MOE_MAX_EXPERTS || N1 < 1 || N2 < 1 || max_rows_per_expert < 0)
    return fail(MOE_ERR_INVALID_ARG, "moe_expert_wgrad: bad shape");
  return launch_wgrad_bf16((const uint16_t*)a, (const uint16_t*)b, expert_offsets, c, c_dtype, a_column_sums, E, N1, N2,
                           max_rows_per_expert, (hipStream_t)stream);
}
