// Bench helper, built into its own small library (libst_bench_probe.so), NOT part of the convolution library
// or its C ABI: what this chip reaches on a plain device-memory copy and on a register-only MFMA loop, to set
// beside the published peaks that the benchmark's roofline is priced against.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

// Four independent 32x32 accumulators per wavefront, operands never change: nothing but the matrix pipe limits it.
// KIND 0: bf16 32x32x16, 1: f16 32x32x16, 2: fp32 as four 32x32x2 (the same 16 bytes of K per lane).
template <int KIND>
__global__ __launch_bounds__(kThreads) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  const uint32_t seed = 0x3c003c00u + threadIdx.x;          // small finite values in every format
  const u32x4 a = {seed, seed, seed, seed}, b = {seed ^ 1u, seed, seed, seed};
  f32x16 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if constexpr (KIND == 0)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[u], 0, 0, 0);
      else if constexpr (KIND == 1)
        acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc[u], 0, 0, 0);
      else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a[j]), __builtin_bit_cast(float, b[j]), acc[u], 0, 0, 0);
      }
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += acc[u][e];
  sink[(size_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

void launch_mfma(int kind, int wgs, float* sink, int iters) {
  const dim3 grid((unsigned)wgs), block(kThreads);
  if (kind == 0) hipLaunchKernelGGL(probe_mfma_kernel<0>, grid, block, 0, nullptr, sink, iters);
  else if (kind == 1) hipLaunchKernelGGL(probe_mfma_kernel<1>, grid, block, 0, nullptr, sink, iters);
  else hipLaunchKernelGGL(probe_mfma_kernel<2>, grid, block, 0, nullptr, sink, iters);
}

}  // namespace

// what 0: device-memory copy, bytes read plus bytes written per second (1 GiB to 1 GiB, far larger than the
// memory-side cache); 1 / 2 / 3: matrix-core FLOP/s of the register-only loop for bf16 / f16 / f32 inputs, two
// 256-thread workgroups on each of the 256 compute units.  Synchronous on the null stream; allocates and frees its
// own buffers.  Returns 0 on success, else the hipError_t.
extern "C" int st_bench_probe_chip(int what, double* rate) {
  if (!rate || what < 0 || what > 3) return (int)hipErrorInvalidValue;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  float ms = 0.f;
  double work = 0.0;
  void* bufs[2] = {nullptr, nullptr};
  const int reps = 5;
  if (what == 0) {
    const int64_t bytes = (int64_t)1 << 30, n16 = bytes / 16;
    if (e == hipSuccess) e = hipMalloc(&bufs[0], (size_t)bytes);
    if (e == hipSuccess) e = hipMalloc(&bufs[1], (size_t)bytes);
    if (e == hipSuccess) e = hipMemset(bufs[0], 1, (size_t)bytes);
    if (e == hipSuccess) {
      hipLaunchKernelGGL(probe_copy_kernel, dim3(8192), dim3(256), 0, nullptr, (const u32x4*)bufs[0], (u32x4*)bufs[1], n16);   // warm-up
      e = hipEventRecord(e0, nullptr);
    }
    for (int r = 0; r < reps && e == hipSuccess; ++r) {
      hipLaunchKernelGGL(probe_copy_kernel, dim3(8192), dim3(256), 0, nullptr, (const u32x4*)bufs[0], (u32x4*)bufs[1], n16);
      e = hipGetLastError();
    }
    work = 2.0 * (double)bytes * reps;
  } else {
    const int wgs = 2 * 256, iters = 4096;
    if (e == hipSuccess) e = hipMalloc(&bufs[0], (size_t)wgs * kThreads * 4);
    if (e == hipSuccess) {
      launch_mfma(what - 1, wgs, (float*)bufs[0], 64);       // warm-up
      e = hipEventRecord(e0, nullptr);
    }
    for (int r = 0; r < reps && e == hipSuccess; ++r) {
      launch_mfma(what - 1, wgs, (float*)bufs[0], iters);
      e = hipGetLastError();
    }
    const double per_call = 2.0 * 32 * 32 * (what == 3 ? 8 : 16);
    work = (double)reps * wgs * (kThreads / 64) * iters * 4.0 * per_call;
  }
  if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  *rate = work / ((double)ms * 1e-3);
  return 0;
}
