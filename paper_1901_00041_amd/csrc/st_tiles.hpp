// Device code shared by the convolution kernels: MFMA wrappers, the tile epilogue, the implicit-GEMM workgroup
// tile (conv_tile), the row tile for few-channel layers (conv_tile_rows) and the per-workgroup dispatch on
// (dtype, tile shape).  Included by st_kernels.hip (one launch per plan) and st_chain.hip (one persistent launch
// over a whole chain of layers).
//
// One workgroup computes one MT x NT output tile (or one split-K slice of it) of one tenant's layer.  The layer is
// the im2col product of Section 4.1 with M = output pixels, N = filters, K = C*R*S; the patch matrix is never
// materialised: each K step gathers a [MT x KB] slab of patches and a [NT x KB] slab of filters into LDS with
// 16-byte loads (NHWC / KRSC make the reduction index channel-contiguous), and the 4 wavefronts run bf16/f16/f32
// MFMA blocks on them with fp32 accumulators.
//
// MFMA operand roles: filters are operand A (block rows), pixels operand B (block columns), so each lane ends up
// with runs of 4 consecutive filters of one pixel, which are contiguous in the NHWC output.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

#include "st_internal.h"

namespace st {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


// The thread's index in its workgroup, read afresh wherever a work item starts.  Inside a loop over work items the
// compiler would otherwise compute everything that depends only on the thread index (lane geometry, staging rows of
// every tile shape) once before the loop and keep it alive in registers through all of it.
__device__ __forceinline__ int work_thread_id() {
  int t = (int)threadIdx.x;
  asm volatile("" : "+v"(t));
  __builtin_assume(t >= 0 && t < kThreads);
  return t;
}

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

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// short-circuit "any": f(0) || f(1) || ... || f(N-1), each f called with an integral_constant
template <int... Is, class F>
__device__ __forceinline__ bool static_any_impl(std::integer_sequence<int, Is...>, F&& f) {
  return (f(std::integral_constant<int, Is>{}) || ...);
}
template <int N, class F>
__device__ __forceinline__ bool static_any(F&& f) {
  return static_any_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// nested conditionals: if (n > 0) { f(0); if (n > 1) { f(1); ... } } up to N levels
template <int I, int N, class F>
__device__ __forceinline__ void static_nest_impl(int n, F&& f) {
  if constexpr (I < N) {
    if (n > I) {
      f(std::integral_constant<int, I>{});
      static_nest_impl<I + 1, N>(n, static_cast<F&&>(f));
    }
  }
}
template <int N, class F>
__device__ __forceinline__ void static_nest(int n, F&& f) {
  static_nest_impl<0, N>(n, static_cast<F&&>(f));
}

// ---- output conversion ---------------------------------------------------------------------------
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);     // v_cvt_pk_bf16_f32: round to nearest even
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

// ---- cache-coherent partial-tile traffic for split-K -------------------------------------------------
// Split-K partial tiles travel between workgroups that may sit on different XCDs, whose L2 caches are
// not coherent with each other.  Instead of fences that write back and invalidate a whole L2, the
// partials themselves are stored and loaded with device-scope coherence (sc1: write through / miss
// always), so the only ordering needed is "my stores have completed" before the arrival counter is
// bumped.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
constexpr int kAuxDeviceCoherent = 16;   // sc1
// How a tile reads activations (x and the residual): what another kernel wrote before this launch can be read
// through the caches (PlainActs); what other workgroups of the SAME launch write (the chain kernel) must be read
// with device-scope loads, which never stop at the compute unit's vector cache and take from the L2 only what that
// L2 itself holds newer than memory (CoherentActs).  Outputs are stored write-through either way; filters never
// change during a launch and always go through the caches.
struct PlainActs { static constexpr int kActAux = 0; };
struct CoherentActs { static constexpr int kActAux = kAuxDeviceCoherent; };

// floor(n / d) for 0 <= n < 2^31 with the planner's multiplier m = floor(2^(31+L)/d)+1, L = ceil(log2 d)
__device__ __forceinline__ int fast_div(int n, uint32_t m, int L) {
  return (int)((uint32_t)(((uint64_t)(uint32_t)n * m) >> 31) >> L);
}

constexpr uint32_t kInvalidOffset = 0x80000000u;   // >= num_records of every buffer: the load returns 0

// ---- epilogue shared by all tile kernels: (+ residual) -> ReLU -> cast -> store ---------------------
// The transposed output rows are stored write-through (sc1), so they leave the L2 while the kernel still runs
// instead of waiting in it for the write-back at the end of the kernel, which the next launch on the stream
// would have to sit through.
// acc[i][j] is the MF x MF block at pixels wm0 + i*MF, filters wn0 + j*MF of the tile whose first pixel is
// im2col row m0 and first filter n0; rows at or past m_end are not stored.
// The transposition buffer `smem` holds MT/PASSES pixel rows; with PASSES > 1 the tile is written out in
// that many slices of consecutive pixel rows.
template <int MT, int NT, int BM, int BN, int MF, int PASSES = 1, int CAP = kSmemBytes, class POL = PlainActs, class Acc, class TD>
__device__ __forceinline__ void tile_epilogue(const TD& T, Acc (&acc)[BM][BN], int m0, int m_end, int n0, int wm0,
                                              int wn0, int lrow, int lk, int tid, char* smem, uint64_t* prof = nullptr) {
  constexpr int NG = (MF == 32) ? 4 : 1;
  const bool relu = (T.epilogue & ST_EPI_RELU) != 0u;
  const bool has_res = (T.epilogue & ST_EPI_RESIDUAL) != 0u;
  const int Kf = T.K;
  const bool vec4 = (Kf & 3) == 0;
  if ((Kf & 7) == 0 && T.out_dtype != ST_DT_F32 && !has_res) {
    // 16-bit output without a residual: ReLU and the rounding are applied to the accumulators, and the
    // transposition buffer holds the finished 16-bit values, [pixel][filter], the whole tile at once.  Every
    // lane then moves 16 bytes of one output row from LDS to memory.
    constexpr int PITCHB = NT * 2 + 16;   // bytes per pixel row; the pad spreads the 8-byte writes of 8 pixels over the banks
    static_assert(MT * PITCHB <= CAP, "16-bit output tile does not fit the transposition buffer");
    const bool isbf = (T.out_dtype == ST_DT_BF16);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(T.y, T.y_bytes);
    __syncthreads();                // the buffer (operands, split-K flag, or the previous tile) is no longer read
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const int row = wm0 + i * MF + lrow;
          const int chl = wn0 + j * MF + ((MF == 32) ? (8 * g + 4 * lk) : (4 * lk));
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = acc[i][j][4 * g + e];
            if (relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
          }
          uint2 pk;
          pk.x = isbf ? ((uint32_t)f32_to_bf16_rne(v[0]) | ((uint32_t)f32_to_bf16_rne(v[1]) << 16))
                      : ((uint32_t)f32_to_f16_bits(v[0]) | ((uint32_t)f32_to_f16_bits(v[1]) << 16));
          pk.y = isbf ? ((uint32_t)f32_to_bf16_rne(v[2]) | ((uint32_t)f32_to_bf16_rne(v[3]) << 16))
                      : ((uint32_t)f32_to_f16_bits(v[2]) | ((uint32_t)f32_to_f16_bits(v[3]) << 16));
          *(uint2*)(smem + row * PITCHB + chl * 2) = pk;
        }
    __syncthreads();
    if (prof && tid == 0) prof[7] = __builtin_readcyclecounter();
    constexpr int NV = NT / 8;
    constexpr int IT = (MT * NV + kThreads - 1) / kThreads;
#pragma unroll
    for (int u = 0; u < IT; ++u) {
      const int v = u * kThreads + tid;
      const int row = v / NV, cv = v % NV;
      const int m = m0 + row, ch = n0 + cv * 8;
      const bool ok = (MT * NV % kThreads == 0 || v < MT * NV) & (m < m_end) & (ch < Kf);
      const uint32_t off = ok ? ((uint32_t)m * (uint32_t)Kf + (uint32_t)ch) * 2u : kInvalidOffset;
      const u32x4 d = *(const u32x4*)(smem + (row < MT ? row : 0) * PITCHB + cv * 16);
      __builtin_amdgcn_raw_buffer_store_b128(d, ry, (int)off, 0, kAuxDeviceCoherent);
    }
  } else if ((Kf & 7) == 0) {
    // Transpose through LDS: accumulators go to an fp32 [pixel][filter] tile, then every lane handles 16
    // bytes of one output row, so residual loads and output stores are whole contiguous rows.
    constexpr int PITCH = NT + 4;   // floats; the pad keeps the 16-byte writes of 16 pixels on distinct banks
    constexpr int MP = MT / PASSES; // pixel rows per slice
    static_assert(MT % PASSES == 0 && MP % MF == 0, "slices must hold whole MFMA blocks");
    static_assert(MP * PITCH * 4 <= CAP, "output tile does not fit the transposition buffer");
    float* sC = (float*)smem;
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(T.y, T.y_bytes);
    const __amdgpu_buffer_rsrc_t rr = make_rsrc(has_res ? T.res : T.y, T.y_bytes);
    // Residual vectors are requested before the accumulators are staged, so their latency overlaps the
    // transposition (single-slice tiles only).
    constexpr int IT32 = (MP * (NT / 4) + kThreads - 1) / kThreads, IT16 = (MP * (NT / 8) + kThreads - 1) / kThreads;
    constexpr bool kPrefetchRes = (PASSES == 1);
    u32x4 rpre[kPrefetchRes ? IT32 : 1];
    if (kPrefetchRes && has_res) {
      if (T.out_dtype == ST_DT_F32) {
#pragma unroll
        for (int u = 0; u < IT32; ++u) {
          const int v = u * kThreads + tid;
          const int m = m0 + v / (NT / 4), ch = n0 + (v % (NT / 4)) * 4;
          const bool ok = (MP * (NT / 4) % kThreads == 0 || v < MP * (NT / 4)) & (m < m_end) & (ch < Kf);
          rpre[u] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)(ok ? ((uint32_t)m * (uint32_t)Kf + (uint32_t)ch) * 4u : kInvalidOffset), 0, POL::kActAux);
        }
      } else {
#pragma unroll
        for (int u = 0; u < IT16; ++u) {
          const int v = u * kThreads + tid;
          const int m = m0 + v / (NT / 8), ch = n0 + (v % (NT / 8)) * 8;
          const bool ok = (MP * (NT / 8) % kThreads == 0 || v < MP * (NT / 8)) & (m < m_end) & (ch < Kf);
          rpre[u] = __builtin_amdgcn_raw_buffer_load_b128(rr, (int)(ok ? ((uint32_t)m * (uint32_t)Kf + (uint32_t)ch) * 2u : kInvalidOffset), 0, POL::kActAux);
        }
      }
    }
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
    const int mp0 = m0 + pass * MP;   // first im2col row of this slice
    __syncthreads();                // the buffer (operands, split-K flag, or the previous slice) is no longer read
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const int row = wm0 + i * MF + lrow - pass * MP;
          const int chl = wn0 + j * MF + ((MF == 32) ? (8 * g + 4 * lk) : (4 * lk));
          if (PASSES == 1 || (row >= 0 && row < MP))
            *(f32x4*)(sC + row * PITCH + chl) = f32x4{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        }
    __syncthreads();
    if (prof && tid == 0) prof[7] = __builtin_readcyclecounter();
    // Branch-free read-back: rows past the tile end or filters past K get an out-of-range offset, which
    // drops the store (and makes the residual load return zero).
    if (T.out_dtype == ST_DT_F32) {
      constexpr int NV = NT / 4;
      constexpr int IT = (MP * NV + kThreads - 1) / kThreads;
      constexpr int UB = IT < 4 ? IT : 4;        // vectors in flight per thread (bounds register use)
#pragma unroll
      for (int u0 = 0; u0 < IT; u0 += UB) {
        f32x4 a[UB];
        uint32_t off[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int v = (u0 + u) * kThreads + tid;
          const int row = v / NV, cv = v % NV;
          const int m = mp0 + row, ch = n0 + cv * 4;
          const bool ok = (MP * NV % kThreads == 0 || v < MP * NV) & (m < m_end) & (ch < Kf);
          off[u] = ok ? ((uint32_t)m * (uint32_t)Kf + (uint32_t)ch) * 4u : kInvalidOffset;
          a[u] = *(const f32x4*)(sC + (row < MP ? row : 0) * PITCH + cv * 4);
        }
        if (has_res) {
#pragma unroll
          for (int u = 0; u < UB; ++u)
            a[u] += __builtin_bit_cast(f32x4, kPrefetchRes ? rpre[u0 + u] : __builtin_amdgcn_raw_buffer_load_b128(rr, (int)off[u], 0, POL::kActAux));
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          if (relu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) a[u][e] = a[u][e] > 0.f ? a[u][e] : 0.f;
          }
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, a[u]), ry, (int)off[u], 0, kAuxDeviceCoherent);
        }
      }
    } else {
      constexpr int NV = NT / 8;
      constexpr int IT = (MP * NV + kThreads - 1) / kThreads;
      constexpr int UB = IT < 4 ? IT : 4;
      const bool isbf = (T.out_dtype == ST_DT_BF16);
#pragma unroll
      for (int u0 = 0; u0 < IT; u0 += UB) {
        f32x4 lo[UB], hi[UB];
        uint32_t off[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int v = (u0 + u) * kThreads + tid;
          const int row = v / NV, cv = v % NV;
          const int m = mp0 + row, ch = n0 + cv * 8;
          const bool ok = (MP * NV % kThreads == 0 || v < MP * NV) & (m < m_end) & (ch < Kf);
          off[u] = ok ? ((uint32_t)m * (uint32_t)Kf + (uint32_t)ch) * 2u : kInvalidOffset;
          const float* src = sC + (row < MP ? row : 0) * PITCH + cv * 8;
          lo[u] = *(const f32x4*)src;
          hi[u] = *(const f32x4*)(src + 4);
        }
        if (has_res) {
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const u32x4 r = kPrefetchRes ? rpre[u0 + u] : __builtin_amdgcn_raw_buffer_load_b128(rr, (int)off[u], 0, POL::kActAux);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const uint16_t h0 = (uint16_t)(r[e >> 1] >> (16 * (e & 1))), h1 = (uint16_t)(r[2 + (e >> 1)] >> (16 * (e & 1)));
              lo[u][e] += isbf ? bf16_bits_to_f32(h0) : f16_bits_to_f32(h0);
              hi[u][e] += isbf ? bf16_bits_to_f32(h1) : f16_bits_to_f32(h1);
            }
          }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          if (relu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              lo[u][e] = lo[u][e] > 0.f ? lo[u][e] : 0.f;
              hi[u][e] = hi[u][e] > 0.f ? hi[u][e] : 0.f;
            }
          }
          u32x4 pk;
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            pk[e] = isbf ? ((uint32_t)f32_to_bf16_rne(lo[u][2 * e]) | ((uint32_t)f32_to_bf16_rne(lo[u][2 * e + 1]) << 16))
                         : ((uint32_t)f32_to_f16_bits(lo[u][2 * e]) | ((uint32_t)f32_to_f16_bits(lo[u][2 * e + 1]) << 16));
            pk[2 + e] = isbf ? ((uint32_t)f32_to_bf16_rne(hi[u][2 * e]) | ((uint32_t)f32_to_bf16_rne(hi[u][2 * e + 1]) << 16))
                             : ((uint32_t)f32_to_f16_bits(hi[u][2 * e]) | ((uint32_t)f32_to_f16_bits(hi[u][2 * e + 1]) << 16));
          }
          __builtin_amdgcn_raw_buffer_store_b128(pk, ry, (int)off[u], 0, kAuxDeviceCoherent);
        }
      }
    }
    }   // slices
  } else {
  #pragma unroll
    for (int i = 0; i < BM; ++i) {
      const int m = m0 + wm0 + i * MF + lrow;
      if (m >= m_end) continue;
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
_Pragma("unroll")
              for (int e = 0; e < 4; ++e)
                if (e < nv) {
                  if constexpr (POL::kActAux == 0) v[e] += rp[e];
                  else v[e] += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(T.res, T.y_bytes), (int)((uint32_t)(o + e) * 4u), 0, POL::kActAux));
                }
            }
            if (relu)
_Pragma("unroll")
              for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
            if (vec4) *(f32x4*)y = f32x4{v[0], v[1], v[2], v[3]};
            else {
_Pragma("unroll")
              for (int e = 0; e < 4; ++e) if (e < nv) y[e] = v[e];
            }
          } else {
            uint16_t* y = (uint16_t*)T.y + o;
            const bool isbf = (T.out_dtype == ST_DT_BF16);
            if (has_res) {
              const uint16_t* rp = (const uint16_t*)T.res + o;
_Pragma("unroll")
              for (int e = 0; e < 4; ++e)
                if (e < nv) {
                  uint16_t rb;
                  if constexpr (POL::kActAux == 0) rb = rp[e];
                  else rb = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(make_rsrc(T.res, T.y_bytes), (int)((uint32_t)(o + e) * 2u), 0, POL::kActAux);
                  v[e] += isbf ? bf16_bits_to_f32(rb) : f16_bits_to_f32(rb);
                }
            }
            if (relu)
_Pragma("unroll")
              for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
            uint16_t hbits[4];
_Pragma("unroll")
            for (int e = 0; e < 4; ++e) hbits[e] = isbf ? f32_to_bf16_rne(v[e]) : f32_to_f16_bits(v[e]);
            if (vec4) {
              uint2 pk;
              pk.x = (uint32_t)hbits[0] | ((uint32_t)hbits[1] << 16);
              pk.y = (uint32_t)hbits[2] | ((uint32_t)hbits[3] << 16);
              *(uint2*)y = pk;
            } else {
_Pragma("unroll")
              for (int e = 0; e < 4; ++e) if (e < nv) y[e] = hbits[e];
            }
          }
        }
    }
  }
}

// ---- one workgroup tile --------------------------------------------------------------------------
// MT x NT output tile, 4 wavefronts as WPX x WCH, MFMA block edge MF, KB bytes of the reduction index
// staged per row per step, D steps of global loads kept in flight in registers ahead of the LDS
// double buffer.  All global loads are buffer loads whose out-of-range lanes return zero, so padding,
// ragged tiles and the end of the K range cost no branches.  GENERIC selects element-wise gathers for
// tensors whose channel count is not a multiple of the 16-byte vector width (e.g. C = 3).
// KW ("K across wavefronts"): instead of dividing the tile's pixels and filters among the four wavefronts (each
// operand row is then read from LDS by WCH resp. WPX of them), every wavefront computes the WHOLE tile over one
// quarter of each K step (sub-step = wavefront index), so every staged byte is read from LDS exactly once.  After
// the K loop the four partial tiles are summed through LDS, in wavefront order, into the accumulators the
// pixel/filter division would have produced, and everything downstream (split-K, epilogue) is unchanged.
template <int MT, int NT, int WPX, int WCH, int MF, int KB, int D, int DT, bool GENERIC, bool KW = false, class POL = PlainActs,
          bool STAP = false, class TD>
__device__ __forceinline__ void conv_tile(const TD& T, const st_work_item it, char* smem, uint64_t* prof) {
  constexpr int ES = ElemOf<DT>::ES;
  constexpr int VEC = 16 / ES;          // elements per 16-byte vector
  constexpr int KT = KB / ES;           // elements of K per step
  constexpr int ROWB = KB + 16;         // LDS row pitch: the 16-byte pad spreads rows over all banks
  constexpr int CH = KB / 16;           // 16-byte chunks per row
  constexpr int RPP = kThreads / CH;    // rows staged per pass of the workgroup
  constexpr int WM = MT / WPX, WN = NT / WCH;
  constexpr int BM = WM / MF, BN = WN / MF;
  constexpr int A_IT = (MT + RPP - 1) / RPP, B_IT = (NT + RPP - 1) / RPP;
  constexpr int SUBB = (MF == 32) ? 32 : 64;   // row bytes one MFMA sub-step consumes
  constexpr int NSUB = KB / SUBB;
  static_assert(D % 2 == 0, "D must be even so that register slots and LDS buffers are both static");
  typedef Mma<DT, MF> MMA;
  typedef typename MMA::Acc Acc;
  static_assert(WPX * WCH == 4 && WM % MF == 0 && WN % MF == 0, "bad tile shape");
  static_assert(2 * (MT + NT) * ROWB <= kSmemBytes, "tile does not fit the LDS allocation");
  constexpr int TBM = MT / MF, TBN = NT / MF;       // MFMA blocks of the whole tile
  static_assert(!KW || (NSUB == 4 && 4 * TBM * TBN * (MF * MF / 64) * 4 * 64 <= kSmemBytes), "KW needs four sub-steps per K step and room for four partial tiles");

  char* sA = smem;                          // [2][MT][ROWB]  patches
  char* sB = smem + 2 * MT * ROWB;          // [2][NT][ROWB]  filters

  const int tid = work_thread_id();
  if (prof && tid == 0) {
    prof[0] = __builtin_readcyclecounter();
    prof[4] = wall_clock64();
    prof[5] = ((uint64_t)__builtin_amdgcn_s_getreg(0x1814) << 32) | (uint32_t)__builtin_amdgcn_s_getreg(0xF804);
  }
  const int chunk = tid % CH;    // which 16 bytes of the row slab this thread stages
  const int row0 = tid / CH;
  const int m0 = (int)it.tile_m * MT;
  const int n0 = (int)it.tile_n * NT;
  const int C = T.C, H = T.H, W = T.W, S = T.S, Kg = T.Kg;
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(T.x, T.x_bytes);
  const __amdgpu_buffer_rsrc_t rw = make_rsrc(T.w, T.w_bytes);

  // K-step range of this work item; loads at or past klimit are suppressed
  const int ks_begin = (int)it.k_split_idx * T.k_steps_per_split;
  int ks_end = ks_begin + T.k_steps_per_split;
  if (ks_end > T.k_steps) ks_end = T.k_steps;
  const int nsteps = ks_end - ks_begin;
  const int klimit = (ks_end * KT < Kg) ? ks_end * KT : Kg;

  // per-thread patch rows
  int a_base[A_IT], a_h0[A_IT], a_w0[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = row0 + i * RPP;
    const int m = m0 + row;
    const bool ok = (row < MT) && (m < T.M);
    const int mm = ok ? m : 0;
    const int n = fast_div(mm, T.magic_pq, T.shift_pq);
    const int pq = mm - n * T.PQ;
    const int p = fast_div(pq, T.magic_q, T.shift_q);
    const int q = pq - p * T.Q;
    a_h0[i] = ok ? p * T.stride - T.pad : -(1 << 24);   // a dead row fails every bounds check
    a_w0[i] = q * T.stride - T.pad;
    a_base[i] = ((n * H + a_h0[i]) * W + a_w0[i]) * C;
  }
  int b_off[B_IT];
  bool b_ok[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int row = row0 + i * RPP;
    b_ok[i] = (row < NT) && (n0 + row < T.K);
    b_off[i] = b_ok[i] ? (n0 + row) * Kg : 0;
  }

  // position of the next vector this thread will fetch, in the reduction index k = (r*S + s)*C + c
  int k_elem = ks_begin * KT + chunk * VEC;
  int k_step0 = ks_begin * KT;   // first element of the step, uniform over the workgroup

  u32x4 ra[D][A_IT], rb[D][B_IT];

  // Issue the global loads of the next K step into one register slot, then advance the K position.
  auto issue = [&](u32x4 (&qa)[A_IT], u32x4 (&qb)[B_IT]) {
    if constexpr (!GENERIC) {
      const bool kin = k_elem < klimit;
      // filter tap (kr, ksx) and offset of this thread's vector
      int kr, ksx, koff;
      if (!STAP || !T.tap_uniform) {
        // per-lane form.  Without STAP this is the only form and a K step is a single basic block: the compiler then
        // overlaps the address arithmetic, the loads and the LDS writes with the MFMAs, which is what a workgroup
        // alone on its compute unit needs (a 128x128 workgroup steps 18 % faster, config 5's late layers 3 %).
        const int rs = fast_div(k_elem, T.magic_c, T.shift_c);
        kr = fast_div(rs, T.magic_s, T.shift_s);
        ksx = rs - kr * S;
        koff = (kr * W + ksx) * C + (k_elem - rs * C);
      } else {
        // C is a multiple of the K step: the whole step lies in one filter tap, found with scalar math.  The small
        // tiles of a launch that puts two workgroups on most compute units are instantiated with STAP and take this
        // path (the planner sets tap_uniform for them; the run-time test keeps the step in several basic blocks, and
        // with a second workgroup to fill the gaps that, with the cheaper arithmetic, is the faster arrangement:
        // configs 2 and 3 lose 6-8 % with either form as a single block).
        const int rs = fast_div(k_step0, T.magic_c, T.shift_c);
        kr = fast_div(rs, T.magic_s, T.shift_s);
        ksx = rs - kr * S;
        koff = (kr * W + ksx) * C + (k_step0 - rs * C) + chunk * VEC;
      }
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        const bool ok = kin & ((unsigned)(a_h0[i] + kr) < (unsigned)H) & ((unsigned)(a_w0[i] + ksx) < (unsigned)W);
        const uint32_t off = ok ? (uint32_t)(a_base[i] + koff) * ES : kInvalidOffset;
        qa[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, POL::kActAux);
      }
#pragma unroll
      for (int i = 0; i < B_IT; ++i) {
        const uint32_t off = (b_ok[i] & kin) ? (uint32_t)(b_off[i] + k_elem) * ES : kInvalidOffset;
        qb[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0);
      }
    } else {
      // element-wise gather: every element of the vector has its own (r, s, c)
      uint32_t ea[A_IT][VEC], eb[B_IT][VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int ke = k_elem + e;
        const bool kin = ke < klimit;
        const int rs = fast_div(ke, T.magic_c, T.shift_c);
        const int kc = ke - rs * C;
        const int kr = fast_div(rs, T.magic_s, T.shift_s);
        const int ksx = rs - kr * S;
        const int koff = (kr * W + ksx) * C + kc;
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
          const bool ok = kin & ((unsigned)(a_h0[i] + kr) < (unsigned)H) & ((unsigned)(a_w0[i] + ksx) < (unsigned)W);
          const uint32_t off = ok ? (uint32_t)(a_base[i] + koff) * ES : kInvalidOffset;
          if constexpr (ES == 4) ea[i][e] = __builtin_amdgcn_raw_buffer_load_b32(rx, (int)off, 0, POL::kActAux);
          else ea[i][e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, (int)off, 0, POL::kActAux);
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
          const uint32_t off = (b_ok[i] & kin) ? (uint32_t)(b_off[i] + ke) * ES : kInvalidOffset;
          if constexpr (ES == 4) eb[i][e] = __builtin_amdgcn_raw_buffer_load_b32(rw, (int)off, 0, 0);
          else eb[i][e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rw, (int)off, 0, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        if constexpr (ES == 4) qa[i] = u32x4{ea[i][0], ea[i][1], ea[i][2], ea[i][3]};
        else qa[i] = u32x4{ea[i][0] | (ea[i][1] << 16), ea[i][2] | (ea[i][3] << 16), ea[i][4] | (ea[i][5] << 16), ea[i][6] | (ea[i][7] << 16)};
      }
#pragma unroll
      for (int i = 0; i < B_IT; ++i) {
        if constexpr (ES == 4) qb[i] = u32x4{eb[i][0], eb[i][1], eb[i][2], eb[i][3]};
        else qb[i] = u32x4{eb[i][0] | (eb[i][1] << 16), eb[i][2] | (eb[i][3] << 16), eb[i][4] | (eb[i][5] << 16), eb[i][6] | (eb[i][7] << 16)};
      }
    }
    k_elem += KT;
    k_step0 += KT;
  };
  auto store_lds = [&](const u32x4 (&qa)[A_IT], const u32x4 (&qb)[B_IT], int buf) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int row = row0 + i * RPP;
      if (MT % RPP == 0 || row < MT) *(u32x4*)(sA + (buf * MT + row) * ROWB + chunk * 16) = qa[i];
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = row0 + i * RPP;
      if (NT % RPP == 0 || row < NT) *(u32x4*)(sB + (buf * NT + row) * ROWB + chunk * 16) = qb[i];
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
  // KW: this wavefront's partial sums of the whole tile
  Acc part[KW ? TBM : 1][KW ? TBN : 1];
  if constexpr (KW) {
#pragma unroll
    for (int i = 0; i < TBM; ++i)
#pragma unroll
      for (int j = 0; j < TBN; ++j)
#pragma unroll
        for (int v = 0; v < (int)(sizeof(Acc) / 4); ++v) part[i][j][v] = 0.f;
  }

  auto compute = [&](int buf) {
    if constexpr (KW) {
      const char* pa = sA + (buf * MT + lrow) * ROWB + lk * 16 + wave * SUBB;
      const char* pb = sB + (buf * NT + lrow) * ROWB + lk * 16 + wave * SUBB;
      u32x4 wf[TBN], xf[TBM];
#pragma unroll
      for (int j = 0; j < TBN; ++j) wf[j] = *(const u32x4*)(pb + j * MF * ROWB);
#pragma unroll
      for (int i = 0; i < TBM; ++i) xf[i] = *(const u32x4*)(pa + i * MF * ROWB);
#pragma unroll
      for (int i = 0; i < TBM; ++i)
#pragma unroll
        for (int j = 0; j < TBN; ++j) part[i][j] = MMA::run(wf[j], xf[i], part[i][j]);
      return;
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
  };

  if (nsteps > 0) {
    // Steps 0..D-1 go in flight at once; step s lives in register slot s % D.  Steps past the end of the
    // K range load nothing (every lane out of range), so no issue below needs a condition.
    static_for<D>([&](auto J) { issue(ra[decltype(J)::value], rb[decltype(J)::value]); });
    store_lds(ra[0], rb[0], 0);
    issue(ra[0], rb[0]);
    __syncthreads();
    if (prof && tid == 0) prof[1] = __builtin_readcyclecounter();
    // one K step: compute from LDS buffer j&1, meanwhile move step k+1 from its register slot to the
    // other buffer and put step k+1+D in flight in that slot
    auto step = [&](auto J) {
      constexpr int j = decltype(J)::value;
      constexpr int nslot = (j + 1) % D;
      compute(j & 1);
      store_lds(ra[nslot], rb[nslot], (j + 1) & 1);
      issue(ra[nslot], rb[nslot]);
      __syncthreads();
    };
    int k = 0;
    for (; k + D <= nsteps; k += D) static_for<D>(step);     // whole groups: no exits, exact wait counts
    // remainder (fewer than D steps), nested so that each step is reached only through the previous one
    const int rem = nsteps - k;
    static_nest<D - 1>(rem, step);
  }

  if constexpr (KW) {
    // sum the four wavefronts' partial tiles: each writes all its blocks ([wavefront][block][lane], 16-byte
    // groups), then takes the blocks of its own share of the tile and adds the four copies in wavefront order
    constexpr int VPB = (int)(sizeof(Acc) / 16);           // 16-byte groups per block per lane
    f32x4* red = (f32x4*)smem;
#pragma unroll
    for (int i = 0; i < TBM; ++i)
#pragma unroll
      for (int j = 0; j < TBN; ++j)
#pragma unroll
        for (int g = 0; g < VPB; ++g)
          red[((wave * TBM * TBN + i * TBN + j) * VPB + g) * 64 + lane] =
              f32x4{part[i][j][4 * g], part[i][j][4 * g + 1], part[i][j][4 * g + 2], part[i][j][4 * g + 3]};
    __syncthreads();
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j) {
        const int bi = wm0 / MF + i, bj = wn0 / MF + j;
#pragma unroll
        for (int g = 0; g < VPB; ++g) {
          f32x4 sum = red[((0 * TBM * TBN + bi * TBN + bj) * VPB + g) * 64 + lane];
#pragma unroll
          for (int w = 1; w < 4; ++w) sum += red[((w * TBM * TBN + bi * TBN + bj) * VPB + g) * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = sum[e];
        }
      }
    __syncthreads();      // the partial tiles are consumed before the epilogue reuses the buffer
  }

  if (prof && tid == 0) prof[2] = __builtin_readcyclecounter();

  // ---- split-K: publish the partial tile; the last workgroup to arrive sums all slices in order --
  constexpr int NG = (MF == 32) ? 4 : 1;      // groups of 4 consecutive filters per block per lane
  if (T.split_k > 1) {
    const int tile_id = (int)it.tile_m * T.tiles_n + (int)it.tile_n;
    constexpr uint32_t kTileBytes = MT * NT * 4;
    const __amdgpu_buffer_rsrc_t rs =
        make_rsrc(T.ws + (int64_t)tile_id * T.split_k * (MT * NT), (uint32_t)T.split_k * kTileBytes);
    const uint32_t my = (uint32_t)it.k_split_idx * kTileBytes;
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rs,
                                                 (((i * BN + j) * NG + g) * kThreads + tid) * 16, my, kAuxDeviceCoherent);
        }
    __builtin_amdgcn_s_waitcnt(0);       // every store of this thread has completed (written through)
    __syncthreads();
    uint32_t* flag = (uint32_t*)smem;
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(&T.counters[tile_id], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t last = (old == (uint32_t)(T.split_k - 1));
      if (last) __hip_atomic_store(&T.counters[tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next run
      *flag = last;
    }
    __syncthreads();
    if (*flag == 0u) {
      if (prof && tid == 0) prof[6] = wall_clock64();
      return;
    }
    // Sum the slices in index order.  Loads are issued in batches (GB groups x SB slices) so that the
    // device-coherent reads, each a trip to memory, overlap; slices past split_k read as zero.
    constexpr int NGRP = BM * BN * NG;
    constexpr int GB = NGRP < 4 ? NGRP : 4;
    constexpr int SB = (NGRP > 4) ? 4 : 8;   // at most 32 partial vectors (128 registers) in flight
    static_assert(NGRP % GB == 0, "group batching");
    const int split = T.split_k;
#pragma unroll
    for (int g0 = 0; g0 < NGRP; g0 += GB) {
      f32x4 sum[GB];
#pragma unroll
      for (int gg = 0; gg < GB; ++gg) sum[gg] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int s0 = 0; s0 < split; s0 += SB) {
        u32x4 part[SB][GB];
#pragma unroll
        for (int ss = 0; ss < SB; ++ss)
#pragma unroll
          for (int gg = 0; gg < GB; ++gg) {
            const uint32_t voff = (s0 + ss < split) ? (uint32_t)(((g0 + gg) * kThreads + tid) * 16) : kInvalidOffset;
            part[ss][gg] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, (s0 + ss) * (int)kTileBytes, kAuxDeviceCoherent);
          }
#pragma unroll
        for (int ss = 0; ss < SB; ++ss)
#pragma unroll
          for (int gg = 0; gg < GB; ++gg) sum[gg] += __builtin_bit_cast(f32x4, part[ss][gg]);
      }
#pragma unroll
      for (int gg = 0; gg < GB; ++gg) {
        constexpr int dummy = 0; (void)dummy;
        const int grp = g0 + gg;
        const int i = grp / (BN * NG), j = (grp / NG) % BN, g = grp % NG;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = sum[gg][e];
      }
    }
  }

  // ---- epilogue: (+ residual) -> ReLU -> cast -> store ---------------------------------------------
  tile_epilogue<MT, NT, BM, BN, MF, 1, kSmemBytes, POL>(T, acc, m0, T.M, n0, wm0, wn0, lrow, lk, tid, smem, prof);
  if (prof && tid == 0) {
    prof[3] = __builtin_readcyclecounter();
    prof[6] = wall_clock64();
  }
}

// The 128 bits that start kk 16-bit elements into the 256-bit value hi:lo (kk wave-uniform, 0..8).
__device__ __forceinline__ u32x4 window128(const u32x4& lo, const u32x4& hi, int kk) {
  const uint32_t b = (uint32_t)(kk & 1) * 16u;
  uint32_t w0, w1, w2, w3, w4;
  switch (kk >> 1) {
    case 0: w0 = lo[0]; w1 = lo[1]; w2 = lo[2]; w3 = lo[3]; w4 = hi[0]; break;
    case 1: w0 = lo[1]; w1 = lo[2]; w2 = lo[3]; w3 = hi[0]; w4 = hi[1]; break;
    case 2: w0 = lo[2]; w1 = lo[3]; w2 = hi[0]; w3 = hi[1]; w4 = hi[2]; break;
    case 3: w0 = lo[3]; w1 = hi[0]; w2 = hi[1]; w3 = hi[2]; w4 = hi[3]; break;
    default: w0 = hi[0]; w1 = hi[1]; w2 = hi[2]; w3 = hi[3]; w4 = 0u; break;
  }
  return u32x4{__builtin_amdgcn_alignbit(w1, w0, b), __builtin_amdgcn_alignbit(w2, w1, b),
               __builtin_amdgcn_alignbit(w3, w2, b), __builtin_amdgcn_alignbit(w4, w3, b)};
}

// ---- row tile for layers with very few input channels ---------------------------------------------
// For the 7x7 / stride-2 / 3-channel stem the im2col row of one (pixel, filter row r) is S*C = 21
// contiguous elements of the NHWC image, at an odd element offset, so neither 16-byte gathers nor the
// element-wise gather variant are efficient.  This kernel gives one workgroup kRowsPerTile consecutive
// output rows (a segment of up to 128 pixels of each) x 64 filters: the input rows they need are copied
// whole into LDS with 16-byte loads (rows outside the image and the left/right padding are zeros), the
// 64 filters are copied once into an LDS array [filter][r][32] padded with zeros, and the MFMA operands
// are assembled from LDS.  K is laid out as r*32 + (s*C + c).  Eligibility is decided by the planner:
// 16-bit types, 8 <= S*C <= 32, W*C*2 a multiple of 16, stride*C even, LDS footprint.
template <int DT, class POL = PlainActs, class TD>
__device__ __forceinline__ void conv_tile_rows(const TD& T, const st_work_item it, char* smem, uint64_t* prof) {
  constexpr int MT = 128, NT = 64, MF = 32, WM = 64, WN = 32, BM = 2, BN = 1, KR = 32;
  const int RT = T.rows_per_tile;                    // output rows per work item (1..kRowsPerTile)
  constexpr int EPI_PASSES = 2;
  // epilogue transposition buffer: the larger of half a tile of fp32 values and a whole tile of 16-bit ones
  constexpr int kStageBytes = kRowStageBytes;
  static_assert(kStageBytes >= (MT / EPI_PASSES) * (NT + 4) * 4 && kStageBytes >= MT * (NT * 2 + 16), "row tile stage buffer");
  typedef Mma<DT, MF> MMA;
  typedef typename MMA::Acc Acc;
  const int tid = work_thread_id();
  if (prof && tid == 0) {
    prof[0] = __builtin_readcyclecounter();
    prof[4] = wall_clock64();
    prof[5] = ((uint64_t)__builtin_amdgcn_s_getreg(0x1814) << 32) | (uint32_t)__builtin_amdgcn_s_getreg(0xF804);
  }
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
  const int lrow = lane & 31, lk = lane >> 5;
  const int C = T.C, H = T.H, W = T.W, R = T.R, S = T.S, P = T.P, Q = T.Q, Kg = T.Kg;
  const int SC = S * C;
  const int qt = (Q + MT - 1) / MT;                 // pixel segments per output row
  const int pg = (P + RT - 1) / RT;                 // row groups per image
  const int npg = (int)it.tile_m / qt;
  const int q0 = ((int)it.tile_m - npg * qt) * MT;
  const int n = npg / pg;
  const int p0 = (npg - n * pg) * RT;
  const int nrows_out = (P - p0 < RT) ? (P - p0) : RT;
  const int n0 = (int)it.tile_n * NT;
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(T.x, T.x_bytes);
  const __amdgpu_buffer_rsrc_t rw = make_rsrc(T.w, T.w_bytes);

  // LDS: [transposition buffer][NR image rows][filters].  Each image row is [pad*C zeros][W*C elements]
  // [zeros] starting on a 16-byte boundary, so that every pixel's patch (which starts stride*C elements
  // after its neighbour's) is 4-byte aligned.
  const int NR = R + T.stride * (RT - 1);                   // input rows held
  const int lpad = T.pad * C * 2;                           // bytes of left padding
  const int rowb = W * C * 2;                               // bytes of one image row (multiple of 16)
  const int pitch = T.row_pitch;                            // bytes of one LDS row (multiple of 16)
  char* sX = smem + kStageBytes;
  char* sW = sX + NR * pitch;                               // [NT][R][KR] elements
  const int h_first = p0 * T.stride - T.pad;

  // Both arrays are written as whole 16-byte vectors in linear order, each from one 16-byte load at a
  // 2-byte-aligned address; a round of 256 filter vectors covers 64 (filter, filter row) pairs with the
  // position inside the filter row fixed per thread.  An image-row vector that straddles an end of the
  // row data, and the last vector of a filter row, are loaded from the nearest position that lies wholly
  // inside the row and shifted into place (zeros move in), so no load touches bytes outside its own row.
  // All loads of the first round are put in flight before the first LDS write.
  const int nvp = pitch >> 4, total_rv = NR * nvp;
  const int sl = (lpad & 15) >> 1;                          // elements the row data sits past a vector boundary
  const int jl = lpad >> 4, jr = (lpad + rowb) >> 4;        // the two straddling vectors of a row (when sl != 0)
  const int nf = (T.K - n0 < NT) ? (T.K - n0) : NT;
  const int nvec = (SC + 7) >> 3;                           // vectors of a filter row that hold data
  const int kkw = 8 * nvec - SC;                            // elements the last of them is loaded early by
  const int npairs = NT * R;                                // (filter, filter row) pairs
  constexpr int RB = 5, RW = 7;                             // rounds per batch: image-row vectors, filter vectors
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  auto row_base = [&](int r) -> uint32_t { return (uint32_t)((n * H + h_first + r) * W) * (uint32_t)(C * 2); };
  auto row_load = [&](int v, bool& mine) -> u32x4 {
    const int r = fast_div(v, T.magic_nvp, T.shift_nvp), j = v - r * nvp;
    const int sj = 16 * j - lpad;                           // byte position of this vector in the row data
    const bool ok = (v < total_rv) & ((unsigned)(h_first + r) < (unsigned)H) & (sj >= 0) & (sj + 16 <= rowb);
    mine = (v < total_rv) & !((sl != 0) & ((j == jl) | (j == jr)));      // the straddlers are written below
    return __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(ok ? row_base(r) + (uint32_t)sj : kInvalidOffset), 0, POL::kActAux);
  };
  auto row_store = [&](int v, const u32x4& d, bool mine) {
    if (mine) *(u32x4*)(sX + v * 16) = d;
  };
  const int slot = tid & 3;                                 // 16-byte position inside a padded filter row
  const bool lastslot = slot == nvec - 1;
  const int e0 = lastslot ? SC - 8 : slot * 8;
  const uint32_t mlast = lastslot ? 0xffffffffu : 0u;
  auto w_load = [&](int cr) -> u32x4 {
    const int ch = fast_div(cr, T.magic_r, T.shift_r), r = cr - ch * R;
    const bool live = (slot < nvec) & (cr < npairs) & (ch < nf);
    const uint32_t off = live ? ((uint32_t)(n0 + ch) * (uint32_t)Kg + (uint32_t)(r * SC + e0)) * 2u : kInvalidOffset;
    return __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0);
  };
  auto w_store = [&](int cr, u32x4 d) {
    if (kkw != 0) {
      const u32x4 ds = window128(d, zero4, kkw);
#pragma unroll
      for (int e = 0; e < 4; ++e) d[e] = (ds[e] & mlast) | (d[e] & ~mlast);
    }
    if (cr < npairs) *(u32x4*)(sW + (cr * 4 + slot) * 16) = d;
  };
  u32x4 drow[RB], dw[RW], dfix = zero4;
  bool rmine[RB];
  const int fr = tid >> 1, fside = tid & 1;                 // straddler (row, end) handled by this thread
#pragma unroll
  for (int u = 0; u < RB; ++u) drow[u] = row_load(u * kThreads + tid, rmine[u]);
  if (sl != 0) {
    const bool ok = (fr < NR) & ((unsigned)(h_first + fr) < (unsigned)H);
    dfix = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(ok ? row_base(fr) + (uint32_t)(fside ? rowb - 16 : 0) : kInvalidOffset), 0, POL::kActAux);
  }
#pragma unroll
  for (int u = 0; u < RW; ++u) dw[u] = w_load((tid >> 2) + 64 * u);
#pragma unroll
  for (int u = 0; u < RB; ++u) row_store(u * kThreads + tid, drow[u], rmine[u]);
  for (int v0 = RB * kThreads; v0 < total_rv; v0 += kThreads) {       // wider images: further rounds
    bool mine;
    const u32x4 d = row_load(v0 + tid, mine);
    row_store(v0 + tid, d, mine);
  }
  if (sl != 0) {
    // left end: the data moves up by sl elements; right end: down by 8 - sl; both are the window that starts
    // 8 - sl elements into (data, zeros) resp. (zeros, data)
    const uint32_t ms = fside ? 0xffffffffu : 0u;
    const u32x4 lo = {dfix[0] & ms, dfix[1] & ms, dfix[2] & ms, dfix[3] & ms};
    const u32x4 hi = {dfix[0] & ~ms, dfix[1] & ~ms, dfix[2] & ~ms, dfix[3] & ~ms};
    const u32x4 d = window128(lo, hi, 8 - sl);
    if (fr < NR) *(u32x4*)(sX + fr * pitch + (fside ? jr : jl) * 16) = d;
  }
#pragma unroll
  for (int u = 0; u < RW; ++u) w_store((tid >> 2) + 64 * u, dw[u]);
  for (int c0 = 64 * RW; c0 < npairs; c0 += 64 * RW) {     // taller filters
#pragma unroll
    for (int u = 0; u < RW; ++u) dw[u] = w_load(c0 + (tid >> 2) + 64 * u);
#pragma unroll
    for (int u = 0; u < RW; ++u) w_store(c0 + (tid >> 2) + 64 * u, dw[u]);
  }
  __syncthreads();
  if (prof && tid == 0) prof[1] = __builtin_readcyclecounter();

  // per-lane masks that clear the elements at or past S*C (they belong to the next pixel)
  uint32_t msk[2][4];
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int j = 16 * half + 8 * lk + 2 * d;
      msk[half][d] = (j < SC ? 0x0000ffffu : 0u) | (j + 1 < SC ? 0xffff0000u : 0u);
    }
  const int nh = (SC + 15) >> 4;     // 16-element halves of a filter row that hold data
  int qa[BM];
#pragma unroll
  for (int i = 0; i < BM; ++i) {
    int q = q0 + wm0 + i * MF + lrow;
    q = q < Q ? q : Q - 1;           // columns past the row end repeat the last pixel; they are never stored
    qa[i] = q * T.stride * C * 2 + lk * 16;
  }
  const char* wrow = sW + (wn0 + lrow) * R * (KR * 2) + lk * 16;
  const int q_end = (q0 + MT < Q) ? q0 + MT : Q;
  // operands of one (filter row, half): the filter vector and BM masked pixel vectors
  struct Ops { u32x4 wf; u32x4 xf[BM]; };
  auto fetch = [&](auto HALF, int rt, int r, Ops& o) {
    constexpr int half = decltype(HALF)::value;
    const char* xr = sX + (rt * T.stride + r) * pitch + half * 32;
    o.wf = *(const u32x4*)(wrow + r * (KR * 2) + half * 32);
#pragma unroll
    for (int i = 0; i < BM; ++i) {
      const uint32_t* src = (const uint32_t*)(xr + qa[i]);
      o.xf[i] = u32x4{src[0], src[1], src[2], src[3]};
    }
  };
  // masking is left to the point of use, so that the LDS reads stay in flight behind the other half's MFMAs
  auto mma = [&](auto HALF, const Ops& o, Acc (&acc)[BM][BN]) {
    constexpr int half = decltype(HALF)::value;
#pragma unroll
    for (int i = 0; i < BM; ++i) {
      const u32x4 xf = {o.xf[i][0] & msk[half][0], o.xf[i][1] & msk[half][1], o.xf[i][2] & msk[half][2], o.xf[i][3] & msk[half][3]};
      acc[i][0] = MMA::run(o.wf, xf, acc[i][0]);
    }
  };
  for (int rt = 0; rt < nrows_out; ++rt) {
    Acc acc[BM][BN];
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][0][v] = 0.f;
    // the operands of the next half step are fetched from LDS while the MFMAs of the current one run; the
    // loop exists once per number of halves so that its body is free of branches
    auto k_loop = [&](auto NH) {
      constexpr int halves = decltype(NH)::value;
      Ops o0, o1;
      fetch(std::integral_constant<int, 0>{}, rt, 0, o0);
      for (int r = 0; r < R; ++r) {
        if constexpr (halves > 1) fetch(std::integral_constant<int, 1>{}, rt, r, o1);
        mma(std::integral_constant<int, 0>{}, o0, acc);
        // the last iteration fetches filter row R - 1 again instead of branching around the reads
        fetch(std::integral_constant<int, 0>{}, rt, (r + 1 < R) ? r + 1 : r, o0);
        if constexpr (halves > 1) mma(std::integral_constant<int, 1>{}, o1, acc);
      }
    };
    if (nh > 1) k_loop(std::integral_constant<int, 2>{}); else k_loop(std::integral_constant<int, 1>{});
    const int mrow = (n * P + p0 + rt) * Q;
    tile_epilogue<MT, NT, BM, BN, MF, EPI_PASSES, kStageBytes, POL>(T, acc, mrow + q0, mrow + q_end, n0, wm0, wn0, lrow, lk, tid, smem);
  }
  if (prof && tid == 0) {
    prof[2] = prof[3] = __builtin_readcyclecounter();
    prof[6] = wall_clock64();
  }
}

template <int CFG, int DT, bool GENERIC, bool KW = false, class POL = PlainActs, bool STAP = false, class TD>
__device__ __forceinline__ void run_cfg(const TD& T, const st_work_item it, char* smem, uint64_t* prof) {
  constexpr TileShape s = kTileShapes[CFG];
  conv_tile<s.MT, s.NT, s.WPX, s.WCH, s.MF, s.KB, s.D, DT, GENERIC, KW, POL, STAP>(T, it, smem, prof);
}

// TD is TenantDev, or TenantDev qualified with the constant address space (records that no launch in flight
// modifies: every field read is then a scalar load, however many stores, atomics and barriers surround it).
template <int DT, class POL = PlainActs, class TD>
__device__ __forceinline__ void run_dtype(const TD& T, const st_work_item it, char* smem, uint64_t* prof) {
  if (T.vec_ok) {
    switch (T.cfg) {
      case 0: run_cfg<0, DT, false, false, POL>(T, it, smem, prof); break;
      case 1: run_cfg<1, DT, false, false, POL>(T, it, smem, prof); break;
      case 2: run_cfg<2, DT, false, false, POL>(T, it, smem, prof); break;
      // the three smallest tiles exist with either form of the tap search (see conv_tile)
      case 3:
        if (T.tap_uniform) run_cfg<3, DT, false, false, POL, true>(T, it, smem, prof);
        else run_cfg<3, DT, false, false, POL>(T, it, smem, prof);
        break;
      // the two smallest tiles split each K step across the wavefronts (see KW above) when the planner found
      // the K loop long enough to repay the final sum of the four partial tiles
      case 4:
        if (T.k_across_waves) {
          if (T.tap_uniform) run_cfg<4, DT, false, true, POL, true>(T, it, smem, prof);
          else run_cfg<4, DT, false, true, POL>(T, it, smem, prof);
        } else {
          if (T.tap_uniform) run_cfg<4, DT, false, false, POL, true>(T, it, smem, prof);
          else run_cfg<4, DT, false, false, POL>(T, it, smem, prof);
        }
        break;
      default:
        if (T.k_across_waves) {
          if (T.tap_uniform) run_cfg<5, DT, false, true, POL, true>(T, it, smem, prof);
          else run_cfg<5, DT, false, true, POL>(T, it, smem, prof);
        } else {
          if (T.tap_uniform) run_cfg<5, DT, false, false, POL, true>(T, it, smem, prof);
          else run_cfg<5, DT, false, false, POL>(T, it, smem, prof);
        }
        break;
    }
  } else {
    // few-channel layers: the row tile when the planner found it eligible, else element-wise gathers
    // (which exist for the two tile shapes marked in kGenericCfg)
    if constexpr (DT != ST_DT_F32) {
      if (T.cfg == kRowCfg) { conv_tile_rows<DT, POL>(T, it, smem, prof); return; }
    }
    if (T.cfg == 1) run_cfg<1, DT, true, false, POL>(T, it, smem, prof);
    else run_cfg<3, DT, true, false, POL>(T, it, smem, prof);
  }
}

// ---- max-pool of one output vector (chain kernel) ---------------------------------------------------
// NHWC max-pool, one 16-byte vector of channels of one output pixel: idx counts (n, p, q, channel vector) with the
// channel vector fastest.  Padding never wins; the result is a copy of the winning input's bits.
// AUX: cache policy of the input loads (0: through the caches; kAuxDeviceCoherent: device-scope loads, for an input
// that other workgroups of the same launch wrote); x_bytes < 2^31 is the size of the input.
template <int DT, int AUX = 0>
__device__ __forceinline__ u32x4 maxpool_vector(const void* __restrict__ xv, uint32_t x_bytes, int64_t idx, int H, int W, int C, int P,
                                                int Q, int win, int stride, int pad) {
  constexpr int ES = ElemOf<DT>::ES, VEC = 16 / ES;
  const int CV = C / VEC;
  const int cv = (int)(idx % CV);
  int64_t t = idx / CV;
  const int q = (int)(t % Q);
  t /= Q;
  const int p = (int)(t % P);
  const int n = (int)(t / P);
  float best[VEC];
  uint32_t bits[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) { best[e] = 0.f; bits[e] = 0u; }
  bool any = false;
  // The taps are visited row by row as a plain loop would, but nine at a time: all nine loads are issued before the
  // first is looked at (taps outside the image or past the window get an out-of-range offset and are skipped), so a
  // 3x3 window costs one memory round trip, not nine.
  constexpr int B = 9;
  const __amdgpu_buffer_rsrc_t rx = make_rsrc(xv, x_bytes);
  const int taps = win * win;
  for (int t0 = 0; t0 < taps; t0 += B) {
    u32x4 raw[B];
    bool ok[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int tp = t0 + u;
      const int r = tp / win, sx = tp - r * win;
      const int h = p * stride - pad + r, w = q * stride - pad + sx;
      ok[u] = (tp < taps) & ((unsigned)h < (unsigned)H) & ((unsigned)w < (unsigned)W);
      const int64_t xoff = ((((int64_t)n * H + h) * W + w) * C + (int64_t)cv * VEC) * ES;
      raw[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(ok[u] ? (uint32_t)xoff : kInvalidOffset), 0, AUX);
    }
#pragma unroll
    for (int u = 0; u < B; ++u) {
      if (!ok[u]) continue;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        uint32_t b;
        float v;
        if constexpr (ES == 4) {
          b = raw[u][e];
          v = __builtin_bit_cast(float, b);
        } else {
          b = (raw[u][e >> 1] >> (16 * (e & 1))) & 0xffffu;
          v = (DT == ST_DT_BF16) ? bf16_bits_to_f32((uint16_t)b) : f16_bits_to_f32((uint16_t)b);
        }
        if (!any || v > best[e]) { best[e] = v; bits[e] = b; }
      }
      any = true;
    }
  }
  if constexpr (ES == 4) return u32x4{bits[0], bits[1], bits[2], bits[3]};
  else return u32x4{bits[0] | (bits[1] << 16), bits[2] | (bits[3] << 16), bits[4] | (bits[5] << 16), bits[6] | (bits[7] << 16)};
}

}  // namespace st
