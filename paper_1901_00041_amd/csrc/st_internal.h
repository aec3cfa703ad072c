// Internal types shared by the host planner and the device kernels (not part of the C ABI).
#pragma once
#include <stdint.h>

#include "st_conv.h"

namespace st {

constexpr int kThreads = 256;      // workgroup size of every conv kernel: 4 wavefronts of 64
constexpr int kNumCUs = 256;       // MI355X
constexpr int kNumXCDs = 8;        // workgroup b of a launch runs on XCD b mod 8
constexpr int kProfSlots = 8;      // 64-bit stamps per work item in a profiled launch

// Tile family.  MT = output pixels (rows of the im2col matrix), NT = filters per workgroup tile.
// The 4 wavefronts form a WPX x WCH grid; MF is the MFMA block edge (32 -> 32x32 blocks,
// 16 -> 16x16 blocks); KB = bytes of the reduction index staged per row per K step; D = K steps of
// global loads kept in flight in registers.
struct TileShape {
  int MT, NT, WPX, WCH, MF, KB, D;
};
constexpr int kNumTileCfgs = 7;
constexpr int kRowCfg = 6;         // the row tile for few-channel layers (conv_tile_rows): 128-pixel segments of
                                   // kRowsPerTile consecutive output rows x 64 filters, one filter row per K step
constexpr int kChainPoolCfg = 7;   // chain kernel only: TenantDev.cfg of a max-pool op (not a convolution tile shape)
constexpr int kScalarTapMinItems = 320;   // work items of a launch from which the scalar form of the tap search is used
constexpr int kRowsPerTile = 4;    // most output rows one row-tile work item may take (the planner picks 1, 2 or 4)
constexpr TileShape kTileShapes[kNumTileCfgs] = {
    {128, 128, 2, 2, 32, 128, 2},  // 0: wave tile 64x64
    {128, 64, 2, 2, 32, 128, 2},   // 1: wave tile 64x32
    {64, 128, 2, 2, 32, 128, 2},   // 2: wave tile 32x64
    {64, 64, 2, 2, 32, 128, 4},    // 3: wave tile 32x32
    {32, 64, 2, 2, 16, 256, 2},    // 4: wave tile 16x32
    {16, 64, 1, 4, 16, 256, 2},    // 5: wave tile 16x16
    {128, 64, 2, 2, 32, 64, 2},    // 6: row tile (few input channels), wave tile 64x32
};
constexpr int smem_need(int c) { return 2 * (kTileShapes[c].MT + kTileShapes[c].NT) * (kTileShapes[c].KB + 16); }
constexpr int kSmemBytes = 73728;  // LDS per workgroup: the largest of the family (checked per tile)
constexpr int kRowStageBytes = 18432;   // row tile: LDS set aside for the epilogue's transposition buffer
// tile shapes that also exist as element-wise-gather kernels (channel count not a multiple of the
// 16-byte vector width); the planner maps such tenants onto one of them
constexpr bool kGenericCfg[kNumTileCfgs] = {false, true, false, true, false, false, false};

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
  int32_t tap_uniform;   // 1: each K step lies within one filter tap (C is a multiple of the step) AND the planner
                         //    wants the tap found with scalar arithmetic (small tiles only; see kScalarTapMinItems)
  int32_t shift_c, shift_s;   // floor(n/d) = ((n * magic) >> 31) >> shift, for d = C and d = S
  uint32_t magic_c, magic_s;
  int32_t shift_r, shift_nvp; // same for d = R and d = row_pitch/16 (row tile only)
  uint32_t magic_r, magic_nvp;
  int32_t shift_pq, shift_q;  // same for d = P*Q and d = Q (pixel index -> image, row, column)
  uint32_t magic_pq, magic_q;
  uint32_t x_bytes, w_bytes;  // buffer sizes for bounds-checked loads
  uint32_t y_bytes;           // size of y (and of the residual) in bytes
  int32_t rows_per_tile;      // row tile only: output rows per work item
  int32_t row_pitch;          // row tile only: bytes of one image row in LDS (padding included, multiple of 16)
  int32_t k_across_waves;     // 1: each wavefront computes the whole tile over a quarter of every K step
  // chain kernel only (st_chain.hip); the per-plan kernel ignores them
  int32_t chain_seq;          // sequence whose completion counter this op's work items wait on and bump
  uint32_t chain_need;        // work items of that sequence that must be complete before this op's may start
  // one completion flag per work item (queue per XCD): work item (tile_m, tile_n, slice) of this op owns flag
  // chain_flag_base + (tile_m * tiles_n + tile_n) * split_k + slice; the op may start once the flags
  // [chain_dep_begin, chain_dep_begin + chain_dep_count) of the sequence's previous stage all hold the run's number
  uint32_t chain_flag_base, chain_dep_begin, chain_dep_count;
  uint32_t chain_reserved;
};
static_assert(sizeof(TenantDev) % 8 == 0, "TenantDev must keep pointer alignment in arrays");

// Launchers implemented in st_kernels.hip.  All asynchronous; return the hipError_t as int.
int launch_conv(const TenantDev* tenants_dev, const st_work_item* items_dev, int64_t n_items, void* stream,
                uint64_t* prof_dev);
// Persistent chain launch (st_chain.hip).  ctl / ctl_other: this run's and the next run's control block.  A block is
// ctl_slots slots of kChainCtlStride 32-bit words (256 bytes) with one live word each, so that the words hundreds of
// workgroups poll and bump sit in different cache lines and memory channels: slot kChainCtlAbort the abort flag,
// kChainCtlDone the count of completed work items, kChainCtlHead the head of the one queue, or with queues per XCD
// kChainCtlHead + 2x + k the number of exclusive (k = 0) / shared (k = 1) columns of XCD x drawn so far,
// kChainCtlSeq + s the completion counter of sequence s; kChainRankWords dense words follow the slots (how many
// workgroups have arrived on each compute unit).  n_queues is 1 (entries [0, n_items) claimed one by one) or
// kNumXCDs (colbegin_dev: kNumXCDs * 2 * kChainColumns + 1 column boundaries in device memory; XCD x's exclusive
// columns are x * 2 * kChainColumns + [0, kChainColumns), its shared ones follow).  item_flags / run_number: the
// per-item completion flags and this run's number (queues per XCD only; else nullptr / anything).
constexpr int kChainCtlStride = 64;
constexpr int kChainCtlAbort = 1, kChainCtlDone = 2, kChainCtlHead = 4, kChainCtlSeq = 4 + 2 * kNumXCDs;
constexpr int kChainRankWords = kNumXCDs * 256;   // arrival counts per (XCD, compute unit key), dense, after the slots
constexpr int kChainColumns = kNumCUs / kNumXCDs; // exclusive columns per XCD (one per compute unit), and as many shared
constexpr uint32_t kChainFlagLocalFlags = 4u;     // completion travels through per-item flags in the XCD's own L2
int chain_max_workgroups(int* out_workgroups, int* out_xcds);
int launch_chain(const TenantDev* ops_dev, const st_work_item* items_dev, uint32_t n_items, const uint32_t* colbegin_dev, uint32_t n_queues,
                 uint32_t* ctl, uint32_t* ctl_other, uint32_t ctl_slots, uint32_t* item_flags, uint32_t run_number,
                 uint32_t spin_limit_ticks, uint32_t flags, int grid, void* stream, uint64_t* prof_dev);
int launch_empty(void* stream);
// Allocation-free path: device address of the current GPU's fixed scratch array (looked up on first use per device),
// host bytes -> device through kernel arguments (sizes rounded up to 16 bytes; dst 16-byte aligned), and a zero fill.
constexpr int64_t kNoallocScratchBytes = (int64_t)32 << 20;
int noalloc_scratch(void** out_ptr);
int launch_poke(const void* host_src, int64_t bytes, void* dst_dev, void* stream);
int launch_zero(void* dst_dev, int64_t bytes, void* stream);
int launch_copy(const void* src, void* dst, int64_t bytes, void* stream);
int launch_maxpool(const void* x, void* y, int N, int H, int W, int C, int P, int Q, int win, int stride,
                   int pad, int dtype, void* stream);

}  // namespace st
