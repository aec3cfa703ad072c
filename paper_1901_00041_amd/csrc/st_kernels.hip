// Fused multi-tenant implicit-GEMM convolution for gfx950 (MI355X).
//
// One launch serves every tenant (the "super-kernel" of Section 4): workgroup b reads work item b,
// looks up its tenant record with scalar loads, and computes one MT x NT output tile (or one split-K
// slice of it) of that tenant's layer.  The layer is the im2col product of Section 4.1 with
// M = output pixels, N = filters, K = C*R*S; the patch matrix is never materialised: each K step
// gathers a [MT x 64 B] slab of patches and a [NT x 64 B] slab of filters into LDS with 16-byte
// loads (NHWC / KRSC make the reduction index channel-contiguous), and the 4 wavefronts run
// bf16/f16/f32 MFMA blocks on them with fp32 accumulators.
//
// MFMA operand roles: filters are operand A (block rows), pixels operand B (block columns), so each
// lane ends up with runs of 4 consecutive filters of one pixel, which are contiguous in the NHWC
// output.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "st_internal.h"

namespace st {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KB = kKStepBytes;   // bytes per row per K step
constexpr int ROWB = KB + 16;     // LDS row pitch: the 16-byte pad spreads rows over all banks

template <int DT> struct ElemOf;
template <> struct ElemOf<ST_DT_F32> { static constexpr int ES = 4; };
template <> struct ElemOf<ST_DT_BF16> { static constexpr int ES = 2; };
template <> struct ElemOf<ST_DT_F16> { static constexpr int ES = 2; };

// ---- MFMA wrappers: one call consumes one 16-byte K fragment per lane ----------------------------
template <int DT, int MF> struct Mma;
template <> struct Mma<ST_DT_BF16, 32> {
  typedef f32x16 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<ST_DT_F16, 32> {
  typedef f32x16 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<ST_DT_F32, 32> {
  typedef f32x16 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], c, 0, 0, 0);
    return c;
  }
};
template <> struct Mma<ST_DT_BF16, 16> {
  typedef f32x4 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<ST_DT_F16, 16> {
  typedef f32x4 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<ST_DT_F32, 16> {
  typedef f32x4 Acc;
  static __device__ __forceinline__ Acc run(u32x4 a, u32x4 b, Acc c) {
    f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[j], fb[j], c, 0, 0, 0);
    return c;
  }
};

// ---- output conversion ---------------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
  _Float16 h = (_Float16)f;
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}

// ---- one workgroup tile --------------------------------------------------------------------------
template <int MT, int NT, int WPX, int WCH, int MF, int DT>
__device__ __forceinline__ void conv_tile(const TenantDev& T, const st_work_item it, char* smem) {
  constexpr int ES = ElemOf<DT>::ES;
  constexpr int VEC = 16 / ES;          // elements per 16-byte vector
  constexpr int KT = KB / ES;           // elements of K per step
  constexpr int WM = MT / WPX, WN = NT / WCH;
  constexpr int BM = WM / MF, BN = WN / MF;
  constexpr int A_IT = (MT + 63) / 64, B_IT = (NT + 63) / 64;
  constexpr int SUBB = (MF == 32) ? 32 : 64;   // row bytes one MFMA sub-step consumes
  constexpr int NSUB = KB / SUBB;
  typedef Mma<DT, MF> MMA;
  typedef typename MMA::Acc Acc;
  static_assert(WPX * WCH == 4 && WM % MF == 0 && WN % MF == 0, "bad tile shape");

  char* sA = smem;                          // [2][MT][ROWB]  patches
  char* sB = smem + 2 * MT * ROWB;          // [2][NT][ROWB]  filters

  const int tid = threadIdx.x;
  const int chunk = tid & 3;     // which 16 bytes of the 64-byte row slab this thread stages
  const int row0 = tid >> 2;     // 0..63
  const int m0 = (int)it.tile_m * MT;
  const int n0 = (int)it.tile_n * NT;
  const char* __restrict__ xg = (const char*)T.x;
  const char* __restrict__ wg = (const char*)T.w;
  const int C = T.C, H = T.H, W = T.W, S = T.S, Kg = T.Kg;

  // K-step range of this work item
  const int ks_begin = (int)it.k_split_idx * T.k_steps_per_split;
  int ks_end = ks_begin + T.k_steps_per_split;
  if (ks_end > T.k_steps) ks_end = T.k_steps;

  // per-thread patch rows
  int a_base[A_IT], a_h0[A_IT], a_w0[A_IT];
  bool a_ok[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = row0 + i * 64;
    const int m = m0 + row;
    a_ok[i] = (row < MT) && (m < T.M);
    const int mm = a_ok[i] ? m : 0;
    const int n = mm / T.PQ;
    const int pq = mm - n * T.PQ;
    const int p = pq / T.Q;
    const int q = pq - p * T.Q;
    a_h0[i] = p * T.stride - T.pad;
    a_w0[i] = q * T.stride - T.pad;
    a_base[i] = ((n * H + a_h0[i]) * W + a_w0[i]) * C;
  }
  int b_off[B_IT];
  bool b_ok[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int row = row0 + i * 64;
    b_ok[i] = (row < NT) && (n0 + row < T.K);
    b_off[i] = b_ok[i] ? (n0 + row) * Kg : 0;
  }

  // position of this thread's vector in the reduction index k = (r*S + s)*C + c
  int k_elem = ks_begin * KT + chunk * VEC;
  int kc = k_elem % C;
  int krs = k_elem / C;
  int ks_ = krs % S;
  int kr = krs / S;

  u32x4 ra[A_IT], rb[B_IT];

  auto load_global = [&]() {
    if (T.vec_ok) {
      const bool kin = k_elem < Kg;
      const int koff = (kr * W + ks_) * C + kc;
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        const bool ok = a_ok[i] && kin && (unsigned)(a_h0[i] + kr) < (unsigned)H && (unsigned)(a_w0[i] + ks_) < (unsigned)W;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (ok) v = *(const u32x4*)(xg + (int64_t)(a_base[i] + koff) * ES);
        ra[i] = v;
      }
#pragma unroll
      for (int i = 0; i < B_IT; ++i) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (b_ok[i] && kin) v = *(const u32x4*)(wg + (int64_t)(b_off[i] + k_elem) * ES);
        rb[i] = v;
      }
    } else {
      // generic gather, element by element (C not a multiple of the vector width, e.g. C = 3)
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const int ke = k_elem + e;
          uint32_t bits = 0u;
          if (a_ok[i] && ke < Kg) {
            const int c = ke % C, rs = ke / C;
            const int s = rs % S, r = rs / S;
            const int h = a_h0[i] + r, w = a_w0[i] + s;
            if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
              const char* p = xg + (int64_t)(a_base[i] + (r * W + s) * C + c) * ES;
              bits = (ES == 4) ? *(const uint32_t*)p : (uint32_t)*(const uint16_t*)p;
            }
          }
          if (ES == 4) pk[e] = bits; else pk[e >> 1] |= bits << (16 * (e & 1));
        }
        ra[i] = u32x4{pk[0], pk[1], pk[2], pk[3]};
      }
#pragma unroll
      for (int i = 0; i < B_IT; ++i) {
        uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const int ke = k_elem + e;
          uint32_t bits = 0u;
          if (b_ok[i] && ke < Kg) {
            const char* p = wg + (int64_t)(b_off[i] + ke) * ES;
            bits = (ES == 4) ? *(const uint32_t*)p : (uint32_t)*(const uint16_t*)p;
          }
          if (ES == 4) pk[e] = bits; else pk[e >> 1] |= bits << (16 * (e & 1));
        }
        rb[i] = u32x4{pk[0], pk[1], pk[2], pk[3]};
      }
    }
  };
  auto advance_k = [&]() {
    k_elem += KT;
    kc += KT;
    while (kc >= C) {
      kc -= C;
      if (++ks_ == S) { ks_ = 0; ++kr; }
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int row = row0 + i * 64;
      if (row < MT) *(u32x4*)(sA + (buf * MT + row) * ROWB + chunk * 16) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = row0 + i * 64;
      if (row < NT) *(u32x4*)(sB + (buf * NT + row) * ROWB + chunk * 16) = rb[i];
    }
  };

  // wavefront / lane geometry
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WPX) * WM;
  const int wn0 = (wave / WPX) * WN;
  const int lrow = lane & (MF - 1);
  const int lk = lane / MF;          // 0..1 for 32x32 blocks, 0..3 for 16x16 blocks

  Acc acc[BM][BN];
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j)
#pragma unroll
      for (int v = 0; v < (int)(sizeof(Acc) / 4); ++v) acc[i][j][v] = 0.f;

  if (ks_begin < ks_end) {
    load_global();
    store_lds(0);
    __syncthreads();
    int buf = 0;
    for (int ks = ks_begin; ks < ks_end; ++ks) {
      const bool more = (ks + 1 < ks_end);
      if (more) {
        advance_k();
        load_global();
      }
      const char* pa = sA + (buf * MT + wm0 + lrow) * ROWB + lk * 16;
      const char* pb = sB + (buf * NT + wn0 + lrow) * ROWB + lk * 16;
#pragma unroll
      for (int sub = 0; sub < NSUB; ++sub) {
        u32x4 wf[BN], xf[BM];
#pragma unroll
        for (int j = 0; j < BN; ++j) wf[j] = *(const u32x4*)(pb + j * MF * ROWB + sub * SUBB);
#pragma unroll
        for (int i = 0; i < BM; ++i) xf[i] = *(const u32x4*)(pa + i * MF * ROWB + sub * SUBB);
#pragma unroll
        for (int i = 0; i < BM; ++i)
#pragma unroll
          for (int j = 0; j < BN; ++j) acc[i][j] = MMA::run(wf[j], xf[i], acc[i][j]);
      }
      if (more) store_lds(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
  }

  // ---- split-K: publish the partial tile; the last workgroup to arrive sums all slices in order --
  constexpr int NG = (MF == 32) ? 4 : 1;      // groups of 4 consecutive filters per block per lane
  if (T.split_k > 1) {
    const int tile_id = (int)it.tile_m * T.tiles_n + (int)it.tile_n;
    f32x4* wsb = (f32x4*)(T.ws + ((int64_t)tile_id * T.split_k + it.k_split_idx) * (MT * NT));
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          wsb[((i * BN + j) * NG + g) * kThreads + tid] = v;
        }
    __threadfence();
    __syncthreads();
    uint32_t* flag = (uint32_t*)smem;
    if (tid == 0) {
      const uint32_t old = atomicAdd(&T.counters[tile_id], 1u);
      const uint32_t last = (old == (uint32_t)(T.split_k - 1));
      if (last) atomicExch(&T.counters[tile_id], 0u);   // ready for the next run
      *flag = last;
    }
    __syncthreads();
    if (*flag == 0u) return;
    __threadfence();
    const f32x4* wst = (const f32x4*)(T.ws + (int64_t)tile_id * T.split_k * (MT * NT));
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          f32x4 sum = {0.f, 0.f, 0.f, 0.f};
          for (int s = 0; s < T.split_k; ++s) {
            const f32x4 v = __builtin_nontemporal_load(&wst[(int64_t)s * (MT * NT / 4) + ((i * BN + j) * NG + g) * kThreads + tid]);
            sum += v;
          }
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = sum[e];
        }
  }

  // ---- epilogue: (+ residual) -> ReLU -> cast -> store ---------------------------------------------
  const bool relu = (T.epilogue & ST_EPI_RELU) != 0u;
  const bool has_res = (T.epilogue & ST_EPI_RESIDUAL) != 0u;
  const int Kf = T.K;
  const bool vec4 = (Kf & 3) == 0;
#pragma unroll
  for (int i = 0; i < BM; ++i) {
    const int m = m0 + wm0 + i * MF + lrow;
    if (m >= T.M) continue;
#pragma unroll
    for (int j = 0; j < BN; ++j)
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int ch = n0 + wn0 + j * MF + ((MF == 32) ? (8 * g + 4 * lk) : (4 * lk));
        if (ch >= Kf) continue;
        float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        const int64_t o = (int64_t)m * Kf + ch;
        const int nv = (Kf - ch < 4) ? (Kf - ch) : 4;
        if (T.out_dtype == ST_DT_F32) {
          float* y = (float*)T.y + o;
          if (has_res) {
            const float* rp = (const float*)T.res + o;
            for (int e = 0; e < nv; ++e) v[e] += rp[e];
          }
          if (relu)
            for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
          if (vec4) *(f32x4*)y = f32x4{v[0], v[1], v[2], v[3]};
          else for (int e = 0; e < nv; ++e) y[e] = v[e];
        } else {
          uint16_t* y = (uint16_t*)T.y + o;
          const bool isbf = (T.out_dtype == ST_DT_BF16);
          if (has_res) {
            const uint16_t* rp = (const uint16_t*)T.res + o;
            for (int e = 0; e < nv; ++e) v[e] += isbf ? bf16_bits_to_f32(rp[e]) : f16_bits_to_f32(rp[e]);
          }
          if (relu)
            for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
          uint16_t hbits[4];
          for (int e = 0; e < 4; ++e) hbits[e] = isbf ? f32_to_bf16_rne(v[e]) : f32_to_f16_bits(v[e]);
          if (vec4) {
            uint2 pk;
            pk.x = (uint32_t)hbits[0] | ((uint32_t)hbits[1] << 16);
            pk.y = (uint32_t)hbits[2] | ((uint32_t)hbits[3] << 16);
            *(uint2*)y = pk;
          } else {
            for (int e = 0; e < nv; ++e) y[e] = hbits[e];
          }
        }
      }
  }
}

constexpr int smem_bytes(int cfg) { return 2 * (kTileShapes[cfg].MT + kTileShapes[cfg].NT) * ROWB; }
constexpr int kSmemMax = smem_bytes(0);

template <int CFG, int DT>
__device__ __forceinline__ void run_cfg(const TenantDev& T, const st_work_item it, char* smem) {
  constexpr TileShape s = kTileShapes[CFG];
  conv_tile<s.MT, s.NT, s.WPX, s.WCH, s.MF, DT>(T, it, smem);
}

template <int DT>
__device__ __forceinline__ void run_dtype(const TenantDev& T, const st_work_item it, char* smem) {
  switch (T.cfg) {
    case 0: run_cfg<0, DT>(T, it, smem); break;
    case 1: run_cfg<1, DT>(T, it, smem); break;
    case 2: run_cfg<2, DT>(T, it, smem); break;
    case 3: run_cfg<3, DT>(T, it, smem); break;
    case 4: run_cfg<4, DT>(T, it, smem); break;
    default: run_cfg<5, DT>(T, it, smem); break;
  }
}

__global__ __launch_bounds__(kThreads) void st_conv_kernel(const TenantDev* __restrict__ tenants,
                                                          const st_work_item* __restrict__ items) {
  __shared__ __attribute__((aligned(16))) char smem[kSmemMax];
  const st_work_item it = items[blockIdx.x];
  const TenantDev& T = tenants[it.tenant];
  switch (T.in_dtype) {
    case ST_DT_BF16: run_dtype<ST_DT_BF16>(T, it, smem); break;
    case ST_DT_F16: run_dtype<ST_DT_F16>(T, it, smem); break;
    default: run_dtype<ST_DT_F32>(T, it, smem); break;
  }
}

__global__ void st_empty_kernel() {}

// NHWC max-pool, one thread per output element; padding never wins.
template <int DT>
__global__ __launch_bounds__(256) void st_maxpool_kernel(const void* __restrict__ xv, void* __restrict__ yv, int N, int H,
                                                         int W, int C, int P, int Q, int win, int stride, int pad) {
  const int64_t total = (int64_t)N * P * Q * C;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % C);
  int64_t t = idx / C;
  const int q = (int)(t % Q);
  t /= Q;
  const int p = (int)(t % P);
  const int n = (int)(t / P);
  float best = -__builtin_inff();
  uint32_t best_bits = 0u;
  bool any = false;
  for (int r = 0; r < win; ++r) {
    const int h = p * stride - pad + r;
    if ((unsigned)h >= (unsigned)H) continue;
    for (int s = 0; s < win; ++s) {
      const int w = q * stride - pad + s;
      if ((unsigned)w >= (unsigned)W) continue;
      const int64_t o = (((int64_t)n * H + h) * W + w) * C + c;
      float v;
      uint32_t bits;
      if (DT == ST_DT_F32) {
        v = ((const float*)xv)[o];
        bits = __builtin_bit_cast(uint32_t, v);
      } else {
        bits = ((const uint16_t*)xv)[o];
        v = (DT == ST_DT_BF16) ? bf16_bits_to_f32((uint16_t)bits) : f16_bits_to_f32((uint16_t)bits);
      }
      if (!any || v > best) { best = v; best_bits = bits; any = true; }
    }
  }
  if (DT == ST_DT_F32) ((uint32_t*)yv)[idx] = best_bits;
  else ((uint16_t*)yv)[idx] = (uint16_t)best_bits;
}

int launch_conv(const TenantDev* tenants_dev, const st_work_item* items_dev, int64_t n_items, void* stream) {
  if (n_items <= 0) return 0;
  hipLaunchKernelGGL(st_conv_kernel, dim3((unsigned)n_items), dim3(kThreads), 0, (hipStream_t)stream, tenants_dev, items_dev);
  return (int)hipGetLastError();
}

int launch_empty(void* stream) {
  hipLaunchKernelGGL(st_empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
  return (int)hipGetLastError();
}

int launch_maxpool(const void* x, void* y, int N, int H, int W, int C, int P, int Q, int win, int stride, int pad,
                   int dtype, void* stream) {
  const int64_t total = (int64_t)N * P * Q * C;
  if (total <= 0) return 0;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipStream_t s = (hipStream_t)stream;
  if (dtype == ST_DT_F32)
    hipLaunchKernelGGL(st_maxpool_kernel<ST_DT_F32>, dim3(blocks), dim3(256), 0, s, x, y, N, H, W, C, P, Q, win, stride, pad);
  else if (dtype == ST_DT_BF16)
    hipLaunchKernelGGL(st_maxpool_kernel<ST_DT_BF16>, dim3(blocks), dim3(256), 0, s, x, y, N, H, W, C, P, Q, win, stride, pad);
  else
    hipLaunchKernelGGL(st_maxpool_kernel<ST_DT_F16>, dim3(blocks), dim3(256), 0, s, x, y, N, H, W, C, P, Q, win, stride, pad);
  return (int)hipGetLastError();
}

}  // namespace st
