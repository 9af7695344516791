// Measured peaks of the machine, for the denominators quoted next to the kernels' numbers: a streaming
// copy and a streaming read (HBM), a loop of nothing but bf16 MFMAs (matrix pipes, with the shader clock it
// ran at) and conflict-free 16-byte LDS reads.  Diagnostics only: part of the phase-timing build of the
// library, never of the product library; it allocates its own buffers.
#include "moesys_internal.h"

namespace moesys {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n, unsigned* out) {
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) acc |= src[i];
  if ((acc.x | acc.y | acc.z | acc.w) == 0x12345u) out[0] = 1;  // never true for the zero-filled buffer; keeps the loads
}

// 8 independent accumulators per wavefront; clocks[0..1] of block 0 = shader clocks and 100 MHz ticks of the loop
__global__ __launch_bounds__(512) void mfma_kernel(int iters, float* out, unsigned long long* clocks) {
  f32x16 acc[8];
  for (int i = 0; i < 8; ++i)
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x & 3); b[i] = (__bf16)1.0f; }
  const unsigned long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0;
  for (int i = 0; i < 8; ++i) s += acc[i][0];
  const unsigned long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  if (s == 12345.f) out[0] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) { clocks[0] = c1 - c0; clocks[1] = r1 - r0; }
}

// every lane reads 16 bytes; rows of 128 bytes with the 16-byte chunk XOR-ed with (row/2) mod 8: the
// layout of the GEMM's operand tiles, free of bank conflicts
__global__ __launch_bounds__(512) void lds_kernel(int iters, unsigned* out, unsigned long long* clocks) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[65536];
  for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) ((unsigned*)smem)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, r = lane & 31, c = lane >> 5;
  const int base = r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
  u32x4 acc = {0, 0, 0, 0};
  const unsigned long long c0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += *reinterpret_cast<const u32x4*>(smem + ((base + j * 4096) & 65535));
    asm volatile("" ::: "memory");
  }
  const unsigned long long c1 = __builtin_readcyclecounter();
  if (acc.x + acc.y + acc.z + acc.w == 0x12345u) out[0] = 1;
  if (blockIdx.x == 0 && threadIdx.x == 0) clocks[2] = c1 - c0;
}

}  // namespace
}  // namespace moesys

using namespace moesys;

// out (host, 6 doubles): copy GB/s (read + written bytes), read GB/s, MFMA TFLOP/s, shader clock of the MFMA
// loop in MHz, LDS read bytes per shader clock per CU, number of CUs.
// Loops of nothing but MFMAs on random (or all-zero) bf16 operands held in registers, for the power probe: the rate
// the matrix pipes reach at the board's power limit depends on the instruction and on the operand values.
// KIND 0: v_mfma_f32_32x32x16_bf16, 4 x 2 fragments of two sub-steps (one 128 x 64 wave tile, 32 values of the
// contraction index); KIND 1: v_mfma_f32_16x16x32_bf16, 8 x 4 fragments (the same wave tile and values).
__device__ inline unsigned mix32(unsigned x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16; return x; }
__device__ inline bf16x8 random_fragment(unsigned seed, bool zero) {
  bf16x8 v;
  for (int i = 0; i < 8; ++i) {
    const unsigned h = mix32(seed * 8 + i);  // roughly normal: four uniforms, centred
    const float u = ((h & 255) + ((h >> 8) & 255) + ((h >> 16) & 255) + (h >> 24)) / 256.f - 2.f;
    v[i] = (__bf16)(zero ? 0.f : u);
  }
  return v;
}
typedef float f32x4 __attribute__((ext_vector_type(4)));
template <int KIND>
__global__ __launch_bounds__(512) void mfma_operand_loop(int iters, int zero, float* out) {
  const unsigned tid = blockIdx.x * 512 + threadIdx.x;
  float s = 0.f;
  if constexpr (KIND == 0) {
    f32x16 acc[4][2];
    for (auto& r : acc) for (auto& a : r) for (int v = 0; v < 16; ++v) a[v] = 0.f;
    bf16x8 A[2][4], B[2][2];
    for (int c = 0; c < 2; ++c) {
      for (int i = 0; i < 4; ++i) A[c][i] = random_fragment(tid * 64 + c * 8 + i, zero);
      for (int j = 0; j < 2; ++j) B[c][j] = random_fragment(tid * 64 + 32 + c * 4 + j, zero);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[c][i], B[c][j], acc[i][j], 0, 0, 0);
    }
    for (auto& r : acc) for (auto& a : r) s += a[0] + a[7];
  } else {
    f32x4 acc[8][4];
    for (auto& r : acc) for (auto& a : r) for (int v = 0; v < 4; ++v) a[v] = 0.f;
    bf16x8 A[8], B[4];
    for (int i = 0; i < 8; ++i) A[i] = random_fragment(tid * 64 + i, zero);
    for (int j = 0; j < 4; ++j) B[j] = random_fragment(tid * 64 + 32 + j, zero);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[i], B[j], acc[i][j], 0, 0, 0);
    }
    for (auto& r : acc) for (auto& a : r) s += a[0] + a[3];
  }
  if (s == 12345.678f) out[0] = s;  // never true; keeps the loop
}

extern "C" int32_t moe_hw_peaks(double* out) {
  if (!out) return fail(MOE_ERR_INVALID_ARG, "moe_hw_peaks: out (8 doubles) is NULL");
  hipDeviceProp_t prop;
  int32_t st;
  if ((st = check_hip(hipGetDeviceProperties(&prop, 0), "hipGetDeviceProperties")) != MOE_OK) return st;
  const int cus = prop.multiProcessorCount;
  const size_t bytes = (size_t)1 << 30, n = bytes / 16;
  void *src = nullptr, *dst = nullptr, *small = nullptr;
  if ((st = check_hip(hipMalloc(&src, bytes), "hipMalloc")) != MOE_OK) return st;
  if ((st = check_hip(hipMalloc(&dst, bytes), "hipMalloc")) != MOE_OK) return st;
  if ((st = check_hip(hipMalloc(&small, 4096), "hipMalloc")) != MOE_OK) return st;
  (void)hipMemset(src, 0, bytes);
  (void)hipMemset(small, 0, 4096);
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  float ms = 0.f;
  const int reps = 10;
  hipLaunchKernelGGL(copy_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, (u32x4*)dst, n);
  (void)hipEventRecord(e0, 0);
  for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(copy_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, (u32x4*)dst, n);
  (void)hipEventRecord(e1, 0);
  (void)hipEventSynchronize(e1);
  (void)hipEventElapsedTime(&ms, e0, e1);
  out[0] = 2.0 * bytes * reps / (ms * 1e-3) / 1e9;
  hipLaunchKernelGGL(read_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, n, (unsigned*)small);
  (void)hipEventRecord(e0, 0);
  for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(read_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, n, (unsigned*)small);
  (void)hipEventRecord(e1, 0);
  (void)hipEventSynchronize(e1);
  (void)hipEventElapsedTime(&ms, e0, e1);
  out[1] = (double)bytes * reps / (ms * 1e-3) / 1e9;
  // one launch that reads 256 MiB no cache holds (a 1 GiB copy ran since): what a kernel that reads its input once,
  // in a layer whose GEMMs have replaced the caches' contents, can get
  double cold_ms = 0.0;
  for (int i = 0; i < reps; ++i) {
    hipLaunchKernelGGL(copy_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, (u32x4*)dst, n);
    (void)hipEventRecord(e0, 0);
    hipLaunchKernelGGL(read_kernel, dim3(cus * 16), dim3(256), 0, 0, (const u32x4*)src, n / 4, (unsigned*)small);
    (void)hipEventRecord(e1, 0);
    (void)hipEventSynchronize(e1);
    (void)hipEventElapsedTime(&ms, e0, e1);
    cold_ms += ms;
  }
  out[6] = (double)(bytes / 4) * reps / (cold_ms * 1e-3) / 1e9;
  unsigned long long* clocks = (unsigned long long*)((char*)small + 1024);
  const int iters = 20000;
  hipLaunchKernelGGL(mfma_kernel, dim3(cus), dim3(512), 0, 0, 100, (float*)small, clocks);
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(mfma_kernel, dim3(cus), dim3(512), 0, 0, iters, (float*)small, clocks);
  (void)hipEventRecord(e1, 0);
  (void)hipEventSynchronize(e1);
  (void)hipEventElapsedTime(&ms, e0, e1);
  out[2] = (double)cus * 8 * iters * 8 * 32768.0 / (ms * 1e-3) / 1e12;
  const int lds_iters = 4000;
  hipLaunchKernelGGL(lds_kernel, dim3(cus), dim3(512), 0, 0, lds_iters, (unsigned*)small, clocks);
  unsigned long long h[3] = {0, 0, 0};
  st = check_hip(hipMemcpy(h, clocks, sizeof(h), hipMemcpyDeviceToHost), "hipMemcpy");
  out[3] = h[1] ? (double)h[0] / (double)h[1] * 100.0 : 0.0;
  out[4] = h[2] ? 512.0 * 16 * 8 * lds_iters / (double)h[2] : 0.0;
  out[5] = cus;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(src);
  (void)hipFree(dst);
  (void)hipFree(small);
  if (st != MOE_OK) return st;
  return check_hip(hipGetLastError(), "moe_hw_peaks");
}

// One launch of the MFMA-only loop (kind 0: 32x32x16, 1: 16x16x32; zero != 0: all-zero operands) on every compute unit,
// synchronous; *tflops receives its rate.  Allocates 4 KB on its first call and keeps it.
extern "C" int32_t moe_mfma_operand_loop(int32_t kind, int32_t zero, int32_t iters, double* tflops) {
  if (!tflops || iters < 1 || kind < 0 || kind > 1) return fail(MOE_ERR_INVALID_ARG, "moe_mfma_operand_loop: bad argument");
  static float* out = nullptr;
  int32_t st;
  if (!out && (st = check_hip(hipMalloc(&out, 4096), "hipMalloc")) != MOE_OK) return st;
  hipDeviceProp_t prop;
  if ((st = check_hip(hipGetDeviceProperties(&prop, 0), "hipGetDeviceProperties")) != MOE_OK) return st;
  const int cus = prop.multiProcessorCount;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  (void)hipEventRecord(e0, 0);
  if (kind == 0) hipLaunchKernelGGL(mfma_operand_loop<0>, dim3(cus), dim3(512), 0, 0, iters, zero, out);
  else hipLaunchKernelGGL(mfma_operand_loop<1>, dim3(cus), dim3(512), 0, 0, iters, zero, out);
  (void)hipEventRecord(e1, 0);
  st = check_hip(hipEventSynchronize(e1), "moe_mfma_operand_loop");
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  // flops per wavefront and iteration: 16 MFMAs x 32768 (kind 0) = 32 MFMAs x 16384 (kind 1)
  *tflops = ms > 0.f ? (double)cus * 8 * iters * 16 * 32768.0 / (ms * 1e-3) / 1e12 : 0.0;
  return st;
}
