// Capacity-bounded, order-preserving token-to-expert dispatch.
//
// The paper gives no dispatch algorithm (it names routing and its imbalance,
// Section 1 and Section 4.1); this is the GShard/Switch capacity rule of the
// gates it evaluates (Section 5.2), kept entirely on the device so that no
// count ever travels to the host (the H2D/D2H round trips Section 3.3.1 sets
// out to remove).
//
// Assignment a = j*T + t.  Bookkeeping kernels and one copy kernel:
//   count : per block of DISPATCH_BLOCK assignments, a per-expert histogram
//   scan  : per expert, exclusive scan of the block histograms -> block bases
//           (only for many blocks; with few blocks every assign block sums the
//           histograms before it by itself, which saves a launch)
//   assign: totals -> counts, kept = min(count, C), expert_offsets; each block
//           ranks its assignments per expert in order (wave ballots + cross-wave
//           prefix), slot = block base + rank, row = offset + slot if slot < C
//           else -1
//   gather: one wavefront per token reads x[t] once and writes its <= k rows
//           (skipped by moe_layer_forward, whose first GEMM gathers the rows
//           from x by row_to_assign itself).
// Everything is integer arithmetic or byte copies: results are bit-exact and
// independent of scheduling (no atomics whose order could matter: the LDS
// histogram atomics only add).
#include <atomic>
#include "moesys_internal.h"

// Bookkeeping scratch of moe_dispatch_static, the variant of moe_dispatch for callers that cannot allocate:
// one array per GPU, held from the moment the library's code is loaded on that GPU until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t STATIC_SCRATCH_BYTES = MOE_DISPATCH_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace moesys {
namespace {

constexpr int BT = 256;  // threads per bookkeeping block = assignments per block
static_assert(BT == DISPATCH_BLOCK, "one assignment per thread");
constexpr int FUSED_SCAN_MAX_BLOCKS = 256;  // above this the block bases come from the scan kernel

__device__ __forceinline__ int expert_of(const int32_t* topk_idx, int a, int T, int k) {
  const int j = a / T, t = a - j * T;
  return topk_idx[(size_t)t * k + j];
}

__global__ __launch_bounds__(BT) void dispatch_count_kernel(const int32_t* __restrict__ topk_idx, int T, int k,
                                                            int E, int32_t* __restrict__ block_hist,
                                                            int32_t* __restrict__ clear8) {
  __shared__ int hist[MOE_MAX_EXPERTS];
  if (clear8 && blockIdx.x == 0 && threadIdx.x < 8) clear8[threadIdx.x] = 0;
  for (int e = threadIdx.x; e < E; e += BT) hist[e] = 0;
  __syncthreads();
  const int a = blockIdx.x * DISPATCH_BLOCK + threadIdx.x;
  if (a < T * k) {
    const int e = expert_of(topk_idx, a, T, k);
    if ((unsigned)e < (unsigned)E) atomicAdd(&hist[e], 1);  // an index outside 0..E-1 is ignored (dropped)
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += BT) block_hist[(size_t)blockIdx.x * E + e] = hist[e];
}

// One block; thread e walks expert e's column of block_hist (coalesced across e) and turns it into the
// exclusive prefix; the totals go to the extra row block_hist[nblocks][.].
__global__ __launch_bounds__(MOE_MAX_EXPERTS) void dispatch_scan_kernel(int32_t* __restrict__ block_hist,
                                                                        int nblocks, int E) {
  const int e = threadIdx.x;
  if (e < E) {
    int run = 0;
    for (int b = 0; b < nblocks; ++b) {
      const int h = block_hist[(size_t)b * E + e];
      block_hist[(size_t)b * E + e] = run;  // becomes the block's base slot
      run += h;
    }
    block_hist[(size_t)nblocks * E + e] = run;
  }
}

// prefixed = 1: block_hist holds exclusive prefixes and a totals row (scan kernel ran);
// prefixed = 0: block_hist holds raw histograms and every block sums what it needs itself;
// prefixed = 2: a single block holds every assignment (few tokens): no histogram was made, the block counts its
// own assignments while ranking them, and clears clear8 (nullable) as the count kernel would have.
__global__ __launch_bounds__(BT) void dispatch_assign_kernel(const int32_t* __restrict__ topk_idx, int T, int k,
                                                             int E, int C, const int32_t* __restrict__ block_hist,
                                                             int nblocks, int prefixed,
                                                             int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ a2r, int32_t* __restrict__ r2a,
                                                             int32_t* __restrict__ clear8) {
  constexpr int NW = BT / 64;
  __shared__ int base_s[MOE_MAX_EXPERTS];        // slots of this expert handed out by earlier blocks
  __shared__ int total_s[MOE_MAX_EXPERTS];       // assignments per expert before capacity
  __shared__ int wave_cnt[NW][MOE_MAX_EXPERTS];  // per-wave counts of this block
  __shared__ int off_s[MOE_MAX_EXPERTS + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int e = threadIdx.x; e < E; e += BT) {
    base_s[e] = prefixed == 1 ? block_hist[(size_t)blockIdx.x * E + e] : 0;
    total_s[e] = prefixed == 1 ? block_hist[(size_t)nblocks * E + e] : 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) wave_cnt[w][e] = 0;
  }
  __syncthreads();
  if (prefixed == 0) {
    // integer adds: the sums do not depend on the order the LDS atomics land in
    const int n = nblocks * E;
    for (int i = threadIdx.x; i < n; i += BT) {
      const int b = i / E, e = i - b * E;
      const int h = block_hist[i];
      if (h) {
        atomicAdd(&total_s[e], h);
        if (b < (int)blockIdx.x) atomicAdd(&base_s[e], h);
      }
    }
    __syncthreads();
  }
  auto prefix_offsets = [&]() {
    if (threadIdx.x == 0) {
      int off = 0;
      for (int e = 0; e < E; ++e) {
        off_s[e] = off;
        off += min(total_s[e], C);
      }
      off_s[E] = off;
    }
  };
  if (prefixed != 2) prefix_offsets();
  const int a = blockIdx.x * DISPATCH_BLOCK + threadIdx.x;
  const int e_in = a < T * k ? expert_of(topk_idx, a, T, k) : -1;
  const bool valid = (unsigned)e_in < (unsigned)E;
  const int e = valid ? e_in : -1;
  // rank among the wave's lanes with the same expert, in lane (= assignment) order
  int rank = 0;
  unsigned long long todo = __ballot(valid);
  while (todo) {
    const int leader = __ffsll((long long)todo) - 1;
    const int e0 = __shfl(e, leader, 64);
    const unsigned long long same = __ballot(e == e0);
    if (e == e0) {
      rank = __popcll(same & ((1ull << lane) - 1ull));
      if (lane == leader) wave_cnt[wave][e0] = __popcll(same);
    }
    todo &= ~same;
  }
  __syncthreads();
  if (prefixed == 2) {  // the totals are this block's own counts
    for (int e2 = threadIdx.x; e2 < E; e2 += BT) {
      int n = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) n += wave_cnt[w][e2];
      total_s[e2] = n;
    }
    __syncthreads();
    prefix_offsets();
    __syncthreads();
    if (clear8 && threadIdx.x < 8) clear8[threadIdx.x] = 0;
  }
  if (blockIdx.x == 0)
    for (int i = threadIdx.x; i <= E; i += BT) {
      offsets[i] = off_s[i];
      if (i < E) counts[i] = total_s[i];
    }
  if (valid) {
    int slot = base_s[e] + rank;
#pragma unroll
    for (int w = 0; w < NW; ++w)
      if (w < wave) slot += wave_cnt[w][e];
    const int row = slot < C ? off_s[e] + slot : -1;
    a2r[a] = row;
    if (row >= 0) r2a[row] = a;
  } else if (a < T * k) {
    a2r[a] = -1;
  }
}

// With no assignment at all the tables still have to say so.
__global__ void dispatch_empty_kernel(int E, int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                      int32_t* __restrict__ clear8) {
  if (clear8 && threadIdx.x < 8) clear8[threadIdx.x] = 0;
  for (int i = threadIdx.x; i <= E; i += blockDim.x) {
    offsets[i] = 0;
    if (i < E) counts[i] = 0;
  }
}

// One wavefront per token: read the row once (16 B per lane per step), write it to each kept row.
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const uint4* __restrict__ x, int T, int k,
                                                              int row_vec,  // 16-byte vectors per row
                                                              const int32_t* __restrict__ a2r,
                                                              uint4* __restrict__ xd) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  int rows[MOE_MAX_TOPK];
  bool any = false;
#pragma unroll
  for (int j = 0; j < MOE_MAX_TOPK; ++j) {
    rows[j] = j < k ? a2r[(size_t)j * T + t] : -1;
    any |= rows[j] >= 0;
  }
  if (!any) return;
  const uint4* src = x + (size_t)t * row_vec;
  for (int v = lane; v < row_vec; v += 64) {
    const uint4 val = src[v];
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j)
      if (rows[j] >= 0) xd[(size_t)rows[j] * row_vec + v] = val;
  }
}

}  // namespace

int32_t launch_dispatch(const moe_config* cfg, const void* x, const int32_t* topk_idx, int32_t* counts,
                        int32_t* offsets, int32_t* a2r, int32_t* r2a, void* xd, void* ws, int32_t* clear8,
                        hipStream_t s) {
  const int T = cfg->T, k = cfg->k, E = cfg->E;
  const int C = moe_capacity(cfg);
  const int nblocks = (int)dispatch_blocks(cfg);
  int32_t* block_hist = (int32_t*)ws;  // [nblocks + 1][E]
  if (nblocks == 0) {
    hipLaunchKernelGGL(dispatch_empty_kernel, dim3(1), dim3(256), 0, s, E, counts, offsets, clear8);
    return check_hip(hipGetLastError(), "dispatch launch");
  }
  if (nblocks == 1) {  // few tokens: one kernel counts, ranks and assigns
    hipLaunchKernelGGL(dispatch_assign_kernel, dim3(1), dim3(BT), 0, s, topk_idx, T, k, E, C, block_hist, 1, 2, counts, offsets, a2r,
                       r2a, clear8);
  } else {
    hipLaunchKernelGGL(dispatch_count_kernel, dim3(nblocks), dim3(BT), 0, s, topk_idx, T, k, E, block_hist, clear8);
    const int prefixed = nblocks > FUSED_SCAN_MAX_BLOCKS;
    if (prefixed)
      hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(MOE_MAX_EXPERTS), 0, s, block_hist, nblocks, E);
    hipLaunchKernelGGL(dispatch_assign_kernel, dim3(nblocks), dim3(BT), 0, s, topk_idx, T, k, E, C, block_hist, nblocks,
                       prefixed, counts, offsets, a2r, r2a, (int32_t*)nullptr);
  }
  if (xd) {
    const int row_vec = (int)((size_t)cfg->d_model * elem_size(cfg->dtype) / 16);
    hipLaunchKernelGGL(dispatch_gather_kernel, dim3((T + 3) / 4), dim3(256), 0, s, (const uint4*)x, T, k, row_vec, a2r,
                       (uint4*)xd);
  }
  return check_hip(hipGetLastError(), "dispatch launch");
}

// xd[r] = x[token of row r] from existing tables (the backward pass gathers the rows the bf16 forward pass
// never materialised).
int32_t launch_gather_rows(const moe_config* cfg, const void* x, const int32_t* a2r, void* xd, hipStream_t s) {
  if (cfg->T == 0) return MOE_OK;
  const int row_vec = (int)((size_t)cfg->d_model * elem_size(cfg->dtype) / 16);
  hipLaunchKernelGGL(dispatch_gather_kernel, dim3((cfg->T + 3) / 4), dim3(256), 0, s, (const uint4*)x, cfg->T, cfg->k, row_vec,
                     a2r, (uint4*)xd);
  return check_hip(hipGetLastError(), "gather launch");
}

}  // namespace moesys

using namespace moesys;

extern "C" int32_t moe_dispatch(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                                int32_t* expert_counts, int32_t* expert_offsets, int32_t* assign_to_row,
                                int32_t* row_to_assign, void* xd, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (!expert_counts || !expert_offsets) return fail(MOE_ERR_INVALID_ARG, "moe_dispatch: expert_counts/expert_offsets are NULL");
  if (cfg->T > 0 && (!topk_idx || !assign_to_row || !row_to_assign))
    return fail(MOE_ERR_INVALID_ARG, "moe_dispatch: topk_idx, assign_to_row and row_to_assign must be non-NULL");
  if (cfg->T > 0 && xd && !x) return fail(MOE_ERR_INVALID_ARG, "moe_dispatch: xd given but x is NULL");
  const size_t need = moe_workspace_bytes(cfg, MOE_WS_DISPATCH);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(MOE_ERR_WORKSPACE, "moe_dispatch: workspace needs %zu bytes, 256-byte aligned (got %zu)", need, ws_bytes);
  return launch_dispatch(cfg, x, topk_idx, expert_counts, expert_offsets, assign_to_row, row_to_assign, xd, ws,
                         nullptr, (hipStream_t)stream);
}

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_addr[MAX_DEVICES];  // address of `scratch` on each device, resolved on first use

// Device address of this GPU's copy of `scratch` (every GPU holds its own, at its own address).
int32_t static_scratch(void** out) {
  int dev = -1;
  int32_t st = check_hip(hipGetDevice(&dev), "hipGetDevice");
  if (st != MOE_OK) return st;
  if (dev < 0 || dev >= MAX_DEVICES) return fail(MOE_ERR_UNSUPPORTED, "moe_dispatch_static: device ordinal %d outside 0..%d", dev, MAX_DEVICES - 1);
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    st = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (st != MOE_OK) return st;
    if (!p || ((uintptr_t)p & 255)) return fail(MOE_ERR_HIP, "moe_dispatch_static: scratch symbol resolved to %p", p);
    g_scratch_addr[dev].store(p, std::memory_order_release);  // (two threads racing here store the same address)
  }
  *out = p;
  return MOE_OK;
}
}  // namespace

extern "C" int32_t moe_dispatch_static(const moe_config* cfg, const void* x, const int32_t* topk_idx,
                                       int32_t* expert_counts, int32_t* expert_offsets, int32_t* assign_to_row,
                                       int32_t* row_to_assign, void* xd, void* stream) {
  int32_t st = moe_config_check(cfg);
  if (st != MOE_OK) return st;
  if (!expert_counts || !expert_offsets) return fail(MOE_ERR_INVALID_ARG, "moe_dispatch_static: expert_counts/expert_offsets are NULL");
  if (cfg->T > 0 && (!topk_idx || !assign_to_row || !row_to_assign))
    return fail(MOE_ERR_INVALID_ARG, "moe_dispatch_static: topk_idx, assign_to_row and row_to_assign must be non-NULL");
  if (cfg->T > 0 && xd && !x) return fail(MOE_ERR_INVALID_ARG, "moe_dispatch_static: xd given but x is NULL");
  const size_t need = moe_workspace_bytes(cfg, MOE_WS_DISPATCH);
  if (need > STATIC_SCRATCH_BYTES)
    return fail(MOE_ERR_UNSUPPORTED, "moe_dispatch_static: k*T=%lld assignments over E=%d experts need %zu bytes of scratch, the static "
                "buffer holds %zu (use moe_dispatch with a workspace)", (long long)cfg->k * cfg->T, cfg->E, need, STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if ((st = static_scratch(&ws)) != MOE_OK) return st;
  // every word of the scratch that the kernels read is written first by the same call (per-block histograms,
  // then their prefixes), so nothing has to be cleared; what the previous call left is never looked at
  return launch_dispatch(cfg, x, topk_idx, expert_counts, expert_offsets, assign_to_row, row_to_assign, xd, ws,
                         nullptr, (hipStream_t)stream);
}
