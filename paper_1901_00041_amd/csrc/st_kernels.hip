// Kernels of the fused multi-tenant convolution launch for gfx950 (MI355X) and their launchers.
//
// One launch serves every tenant (the "super-kernel" of Section 4): workgroup b reads work item b, looks up its
// tenant record with scalar loads, and computes one output tile (or one split-K slice of it) of that tenant's layer
// with the tile code of st_tiles.hpp.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cstring>
#include <mutex>
#include <utility>

#include "st_internal.h"
#include "st_tiles.hpp"

// Fixed scratch memory for the entry point that allocates nothing (st_conv_run_noalloc).  One array per GPU, held
// from the moment the code object is loaded on that GPU until the process ends.  Host code never uses the array's
// name as an address: the device address is looked up once per device (st::noalloc_scratch) and kept.
static __device__ __align__(256) unsigned char scratch[st::kNoallocScratchBytes];

namespace st {

__global__ __launch_bounds__(kThreads, 2) void st_conv_kernel(const TenantDev* __restrict__ tenants,
                                                          const st_work_item* __restrict__ items,
                                                          uint64_t* __restrict__ prof_base) {
  __shared__ __attribute__((aligned(16))) char smem[kSmemBytes];
  const st_work_item it = items[blockIdx.x];
  const TenantDev& T = tenants[it.tenant];
  uint64_t* prof = prof_base ? prof_base + (size_t)blockIdx.x * kProfSlots : nullptr;
  switch (T.in_dtype) {
    case ST_DT_BF16: run_dtype<ST_DT_BF16>(T, it, smem, prof); break;
    case ST_DT_F16: run_dtype<ST_DT_F16>(T, it, smem, prof); break;
    default: run_dtype<ST_DT_F32>(T, it, smem, prof); break;
  }
}

__global__ void st_empty_kernel() {}

// NHWC max-pool; padding never wins.  One thread per (output pixel, group of VEC channels): the window's
// 16-byte channel vectors are loaded whole.  VEC = 1 is the fallback for channel counts that are not a
// multiple of the vector width.
template <int DT, int VEC>
__global__ __launch_bounds__(256) void st_maxpool_kernel(const void* __restrict__ xv, void* __restrict__ yv, int N, int H,
                                                         int W, int C, int P, int Q, int win, int stride, int pad) {
  constexpr int ES = (DT == ST_DT_F32) ? 4 : 2;
  const int CV = C / VEC;
  const int64_t total = (int64_t)N * P * Q * CV;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int cv = (int)(idx % CV);
  int64_t t = idx / CV;
  const int q = (int)(t % Q);
  t /= Q;
  const int p = (int)(t % P);
  const int n = (int)(t / P);
  float best[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) best[e] = -__builtin_inff();
  uint32_t bits[VEC];      // bit pattern of the current maximum, so the result is copied, not re-rounded
#pragma unroll
  for (int e = 0; e < VEC; ++e) bits[e] = 0u;
  bool any = false;
  for (int r = 0; r < win; ++r) {
    const int h = p * stride - pad + r;
    if ((unsigned)h >= (unsigned)H) continue;
    for (int s = 0; s < win; ++s) {
      const int w = q * stride - pad + s;
      if ((unsigned)w >= (unsigned)W) continue;
      const char* src = (const char*)xv + ((((int64_t)n * H + h) * W + w) * C + (int64_t)cv * VEC) * ES;
      uint32_t raw[VEC * ES / 4 > 0 ? VEC * ES / 4 : 1];
      if constexpr (VEC * ES == 16) {
        const u32x4 v = *(const u32x4*)src;
        raw[0] = v[0]; raw[1] = v[1]; raw[2] = v[2]; raw[3] = v[3];
      } else if constexpr (ES == 4) {
        raw[0] = *(const uint32_t*)src;
      } else {
        raw[0] = *(const uint16_t*)src;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        uint32_t b;
        float v;
        if constexpr (ES == 4) {
          b = raw[e];
          v = __builtin_bit_cast(float, b);
        } else {
          b = (raw[e >> 1] >> (16 * (e & 1))) & 0xffffu;
          v = (DT == ST_DT_BF16) ? bf16_bits_to_f32((uint16_t)b) : f16_bits_to_f32((uint16_t)b);
        }
        if (!any || v > best[e]) { best[e] = v; bits[e] = b; }
      }
      any = true;
    }
  }
  char* dst = (char*)yv + idx * (int64_t)(VEC * ES);
  if constexpr (VEC * ES == 16) {
    u32x4 o;
    if constexpr (ES == 4) { o = u32x4{bits[0], bits[1], bits[2], bits[3]}; }
    else { o = u32x4{bits[0] | (bits[1] << 16), bits[2] | (bits[3] << 16), bits[4] | (bits[5] << 16), bits[6] | (bits[7] << 16)}; }
    *(u32x4*)dst = o;
  } else if constexpr (ES == 4) {
    *(uint32_t*)dst = bits[0];
  } else {
    *(uint16_t*)dst = (uint16_t)bits[0];
  }
}

int launch_conv(const TenantDev* tenants_dev, const st_work_item* items_dev, int64_t n_items, void* stream,
                uint64_t* prof_dev) {
  if (n_items <= 0) return 0;
  hipLaunchKernelGGL(st_conv_kernel, dim3((unsigned)n_items), dim3(kThreads), 0, (hipStream_t)stream, tenants_dev, items_dev,
                     prof_dev);
  return (int)hipGetLastError();
}

// Plain 16-byte-per-lane copy: the reference kernel for scaling hardware traffic counters.
__global__ __launch_bounds__(256) void st_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

int launch_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  const int64_t n16 = bytes / 16;
  if (n16 <= 0) return 0;
  const unsigned blocks = (unsigned)((n16 + 255) / 256 < 8192 ? (n16 + 255) / 256 : 8192);
  hipLaunchKernelGGL(st_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, n16);
  return (int)hipGetLastError();
}

// ---- the entry point that allocates nothing: tables and split-K workspace in the fixed array `scratch` -------
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Bytes that travel to the device inside the kernel arguments (a launch copies its arguments when it is issued, so
// the host buffer is free again as soon as the launch call returns, and no copy routine is involved).
constexpr int kPokeVecs = 224;                       // 3584 bytes per launch
struct PokePayload { u32x4 v[kPokeVecs]; };
}  // namespace

__global__ __launch_bounds__(256) void st_poke_kernel(PokePayload p, u32x4* __restrict__ dst, int nvec) {
  const int i = threadIdx.x;
  if (i < nvec) dst[i] = p.v[i];
}

__global__ __launch_bounds__(256) void st_zero_kernel(u32x4* __restrict__ dst, int64_t nvec) {
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * blockDim.x) dst[i] = z;
}

int noalloc_scratch(void** out_ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(::scratch));     // this device's copy of the array (the current device's)
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out_ptr = g_scratch_ptr[dev];
  return 0;
}

int launch_poke(const void* host_src, int64_t bytes, void* dst_dev, void* stream) {
  const char* src = (const char*)host_src;
  char* dst = (char*)dst_dev;
  PokePayload p;
  for (int64_t done = 0; done < bytes; done += (int64_t)sizeof(PokePayload)) {
    const int64_t n = bytes - done < (int64_t)sizeof(PokePayload) ? bytes - done : (int64_t)sizeof(PokePayload);
    std::memset(&p, 0, sizeof(p));
    std::memcpy(&p, src + done, (size_t)n);
    hipLaunchKernelGGL(st_poke_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, p, (u32x4*)(dst + done), (int)((n + 15) / 16));
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}

int launch_zero(void* dst_dev, int64_t bytes, void* stream) {
  const int64_t nvec = (bytes + 15) / 16;
  if (nvec <= 0) return 0;
  const unsigned blocks = (unsigned)((nvec + 255) / 256 < 1024 ? (nvec + 255) / 256 : 1024);
  hipLaunchKernelGGL(st_zero_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst_dev, nvec);
  return (int)hipGetLastError();
}

int launch_empty(void* stream) {
  hipLaunchKernelGGL(st_empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
  return (int)hipGetLastError();
}

int launch_maxpool(const void* x, void* y, int N, int H, int W, int C, int P, int Q, int win, int stride, int pad,
                   int dtype, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  const int es = dtype == ST_DT_F32 ? 4 : 2;
  const int vec = (C % (16 / es) == 0) ? 16 / es : 1;
  const int64_t total = (int64_t)N * P * Q * (C / vec);
  if (total <= 0) return 0;
  const unsigned blocks = (unsigned)((total + 255) / 256);
#define ST_POOL(DT, V) \
  hipLaunchKernelGGL((st_maxpool_kernel<DT, V>), dim3(blocks), dim3(256), 0, s, x, y, N, H, W, C, P, Q, win, stride, pad)
  if (dtype == ST_DT_F32) { if (vec == 4) ST_POOL(ST_DT_F32, 4); else ST_POOL(ST_DT_F32, 1); }
  else if (dtype == ST_DT_BF16) { if (vec == 8) ST_POOL(ST_DT_BF16, 8); else ST_POOL(ST_DT_BF16, 1); }
  else { if (vec == 8) ST_POOL(ST_DT_F16, 8); else ST_POOL(ST_DT_F16, 1); }
#undef ST_POOL
  return (int)hipGetLastError();
}

}  // namespace st
