// Internal types shared by the host planner and the device kernels (not part of the C ABI).
#pragma once
#include <stdint.h>

#include "st_conv.h"

namespace st {

constexpr int kThreads = 256;      // workgroup size of every conv kernel: 4 wavefronts of 64
constexpr int kKStepBytes = 64;    // bytes of the reduction dimension staged per row per K step
constexpr int kNumCUs = 256;       // MI355X

// Tile family.  MT = output pixels (rows of the im2col matrix), NT = filters per workgroup tile.
// The 4 wavefronts form a WPX x WCH grid; MF is the MFMA block edge (32 -> 32x32 blocks,
// 16 -> 16x16 blocks).
struct TileShape {
  int MT, NT, WPX, WCH, MF;
};
constexpr int kNumTileCfgs = 6;
constexpr TileShape kTileShapes[kNumTileCfgs] = {
    {128, 128, 2, 2, 32},  // 0: wave tile 64x64
    {128, 64, 2, 2, 32},   // 1: wave tile 64x32
    {64, 128, 2, 2, 32},   // 2: wave tile 32x64
    {64, 64, 2, 2, 32},    // 3: wave tile 32x32
    {32, 64, 2, 2, 16},    // 4: wave tile 16x32
    {16, 64, 1, 4, 16},    // 5: wave tile 16x16
};

// Device-side tenant record, read through scalar loads by every workgroup of that tenant.
struct TenantDev {
  const void* x;
  const void* w;
  void* y;
  const void* res;
  float* ws;             // split-K partial tiles (nullptr when split_k == 1)
  uint32_t* counters;    // one arrival counter per output tile (split-K only), zero between runs
  int32_t C, H, W, K, R, S, stride, pad;
  int32_t P, Q, PQ, M, Kg;
  int32_t in_dtype, out_dtype, epilogue;
  int32_t cfg, split_k, k_steps, k_steps_per_split;
  int32_t tiles_m, tiles_n;
  int32_t vec_ok;        // 1: C is a multiple of the 16-byte vector width, gathers use 16-byte loads
  int32_t pad_;
};
static_assert(sizeof(TenantDev) % 8 == 0, "TenantDev must keep pointer alignment in arrays");

// Launchers implemented in st_kernels.hip.  All asynchronous; return the hipError_t as int.
int launch_conv(const TenantDev* tenants_dev, const st_work_item* items_dev, int64_t n_items, void* stream);
int launch_empty(void* stream);
int launch_maxpool(const void* x, void* y, int N, int H, int W, int C, int P, int Q, int win, int stride,
                   int pad, int dtype, void* stream);

}  // namespace st
