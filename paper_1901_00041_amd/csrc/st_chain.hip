// The fused space-time policy over a whole chain of dependent layers as ONE persistent launch (gfx950).
//
// Section 4 merges the ready kernels of disjoint DNN graphs into super-kernels; a launch per layer still pays, per
// layer, the launch gap, the ramp of a fresh grid and the drain of its slowest tile.  Here every tenant's whole
// sequence of layers sits in one work queue in (stage, cost) order.  A fixed set of resident workgroups claims
// queue entries in order with one atomic each; an entry of sequence q and stage s may start once every work item of
// q's earlier stages is complete (one completion counter per sequence), so a tenant's next layer starts the moment
// its own previous layer is done, while other tenants' tiles fill the slots that its stragglers leave idle.
//
// Progress: entries are claimed strictly in queue order and every entry depends only on entries before it, so the
// lowest unfinished entry is always held by a running workgroup whose dependencies are complete; no co-residency of
// all workgroups is needed.  Every wait is bounded twice over: by a wall-clock limit and by a count of polls; when
// either expires the waiter raises the abort flag, and every workgroup leaves at its next claim or wait.  A workgroup
// also claims at most n_items + 1 times.  So the kernel always exits, whatever the clock or the counters do.
//
// Memory: producers write their outputs through to memory (device-scope stores) and wait for them before they
// signal; consumers read activations, residuals and partial tiles with device-scope loads (CoherentActs), which
// never stop at a vector cache and take from an L2 only what that L2 holds newer than memory, so no cache is ever
// invalidated.  (The workgroup-scope invalidate does nothing for a workgroup that sits on one compute unit, and
// the device-scope one also empties the XCD's L2 of the filters: measured 1-2 us per work item.)  The signal is,
// with one queue for the chip, a device-scope atomic on the sequence's counter; with queues per XCD, where producer
// and consumer share one L2, a plain store of the run's number into the work item's own flag, which the consumer's
// polls then find in that L2 (0.25 us from store to sight, against 0.6 us and more through memory).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

#include "st_internal.h"
#include "st_tiles.hpp"

namespace st {

struct ChainArgs {
  const TenantDev* ops;
  const st_work_item* items;
  uint32_t* ctl;          // this run's control block
  uint32_t* ctl_other;    // the next run's: cleared by workgroup 0
  uint64_t* prof;         // kProfSlots stamps per queue entry, or nullptr
  uint32_t* item_flags;   // kChainFlagLocalFlags: one completion flag per work item, holding the number of the run that set it
  uint32_t run_number;    // this run's number (never 0)
  uint32_t ctl_slots;     // 256-byte slots of a control block (one live word each); kChainRankWords dense words follow them
  uint32_t spin_limit;    // ticks of the 100 MHz constant clock a dependency wait may last
  uint32_t flags;         // kChainFlag*
  uint32_t n_queues;      // 1: one queue for the whole chip, entries claimed one by one; kNumXCDs: columns (see st_chain_kernel)
  uint32_t q_end;         // one queue: it is items[0 .. q_end)
  const uint32_t* colbegin;   // columns: column j of XCD x is items[colbegin[x * 2 * kChainColumns + j] .. colbegin[.. + j + 1])
};

constexpr int kChainGraceLooks = 24;             // looks at a dependency (0.3 us each) before the filter touches are issued
                                                 // (per pass of the 8 x 53-layer chain: 6 looks 459 us, 12: 456, 24 and 48: 454, never touching: 456)
constexpr uint32_t kChainMaxPolls = 1u << 22;   // a poll takes a microsecond or so: seconds, far beyond any real wait

// The op table and the queue never change while a launch runs: they are read through the constant address space, so
// that every field is a scalar load.  (Through plain global pointers nothing counts as invariant inside the loop
// over work items, which has stores, atomics and barriers in it, and every barrier of the tile code forces vector
// re-loads of the op record.)
typedef __attribute__((address_space(4))) const st_work_item ConstItem;
typedef __attribute__((address_space(4))) const TenantDev ConstOp;

template <int DT>
__device__ __forceinline__ void pool_item(ConstOp& T, const st_work_item it) {
  const int64_t idx = (int64_t)it.tile_m * kThreads + work_thread_id();
  if (idx >= (int64_t)T.M) return;
  const u32x4 v = maxpool_vector<DT, kAuxDeviceCoherent>(T.x, T.x_bytes, idx, T.H, T.W, T.C, T.P, T.Q, T.R, T.stride, T.pad);
  __builtin_amdgcn_raw_buffer_store_b128(v, make_rsrc(T.y, T.y_bytes), (int)((uint32_t)idx * 16u), 0, kAuxDeviceCoherent);
}

// One queue entry's work.
__device__ __forceinline__ void chain_item(ConstOp& T, const st_work_item it, char* smem, uint64_t* prof) {
  if (T.cfg == kChainPoolCfg) {
    switch (T.in_dtype) {
      case ST_DT_BF16: pool_item<ST_DT_BF16>(T, it); break;
      case ST_DT_F16: pool_item<ST_DT_F16>(T, it); break;
      default: pool_item<ST_DT_F32>(T, it); break;
    }
  } else {
    switch (T.in_dtype) {
      case ST_DT_BF16: run_dtype<ST_DT_BF16, CoherentActs>(T, it, smem, prof); break;
      case ST_DT_F16: run_dtype<ST_DT_F16, CoherentActs>(T, it, smem, prof); break;
      default: run_dtype<ST_DT_F32, CoherentActs>(T, it, smem, prof); break;
    }
  }
}

// While a work item waits for its sequence's previous stage, its filter slab is pulled towards the compute unit: the
// filters do not depend on any earlier layer, they are read from memory exactly once per pass, and a cold first touch
// from HBM is the longest single latency of a small item.  One 4-byte load per 128-byte line of the rows
// [n0, n0 + NT) x this item's K range; nothing waits for the loads here (the value is consumed after the wait).
__device__ __forceinline__ uint32_t prefetch_filters(ConstOp& T, const st_work_item it, int tid) {
  constexpr int kMaxLoads = 12;                       // per thread: 384 KB per workgroup at most
  const int cfg = T.cfg;
  if (cfg >= kNumTileCfgs || cfg == kRowCfg) return 0u;
  const int NT = kTileShapes[cfg].NT, KB = kTileShapes[cfg].KB;
  const int es = T.in_dtype == ST_DT_F32 ? 4 : 2;
  const int n0 = (int)it.tile_n * NT;
  const int rows = (T.K - n0 < NT) ? (T.K - n0) : NT;
  const int row_bytes = T.Kg * es;
  int kb0 = (int)it.k_split_idx * T.k_steps_per_split * KB;
  int kb1 = kb0 + T.k_steps_per_split * KB;
  if (kb1 > row_bytes) kb1 = row_bytes;
  if (rows <= 0 || kb1 <= kb0) return 0u;
  const int lines_per_row = (kb1 - kb0 + 127) >> 7;
  const int total = rows * lines_per_row;
  const __amdgpu_buffer_rsrc_t rw = make_rsrc(T.w, T.w_bytes);
  uint32_t acc = 0u;
#pragma unroll
  for (int u = 0; u < kMaxLoads; ++u) {
    const int l = u * kThreads + tid;
    const int r = l / lines_per_row, c = l - r * lines_per_row;
    const uint32_t off = (l < total) ? (uint32_t)((n0 + r) * row_bytes + kb0 + (c << 7)) : kInvalidOffset;
    acc |= (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rw, (int)off, 0, 0);
  }
  return acc;
}

// Next position of queue q for this workgroup (thread 0 only); past the end once the pass has been abandoned.
__device__ __forceinline__ uint32_t chain_claim(const ChainArgs& a, uint32_t q, uint32_t qb, uint32_t qe) {
  uint32_t idx = qb + __hip_atomic_fetch_add(&a.ctl[(kChainCtlHead + q) * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (idx >= qe || __hip_atomic_load(&a.ctl[kChainCtlAbort * kChainCtlStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) idx = 0xffffffffu;
  return idx;
}

// With queues per XCD, an XCD's entries are dealt into 2 x kChainColumns COLUMNS, each a list of entries in stage
// order, and every workgroup works through ONE column that it draws when it starts (one atomic): nothing is claimed
// per entry, so no round trip to memory stands between a finished entry and the workgroup's next one.  Two
// workgroups fit a compute unit, and two tiles that share one run 20-45 % slower each than a tile that has it to
// itself; a stage of a sequence often has no more tiles than the XCD has compute units.  So the first workgroup to
// arrive on a compute unit draws one of the kChainColumns EXCLUSIVE columns and every later one a SHARED column, and
// the host deals a stage's entries (longest first) to the exclusive columns first, to the shared ones only beyond
// one per compute unit.  Every column that holds entries needs a workgroup: should fewer become resident on an XCD
// than it has columns in use, the entries of the columns nobody drew stay undone, their dependants' waits expire,
// and the pass is abandoned and reported.  (The one-queue form, whose entries are claimed one by one, completes with
// any number of resident workgroups.)
__global__ __launch_bounds__(kThreads, 2) void st_chain_kernel(const ChainArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[kSmemBytes];
  __shared__ uint32_t s_msg[2];
  const int tid = threadIdx.x;
  if (blockIdx.x == 0) {
    // the control block of the NEXT run (runs alternate between two blocks; the stream orders them)
    for (uint32_t i = (uint32_t)tid; i < a.ctl_slots; i += kThreads)
      __hip_atomic_store(&a.ctl_other[i * kChainCtlStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (uint32_t i = (uint32_t)tid; i < (uint32_t)kChainRankWords; i += kThreads)
      __hip_atomic_store(&a.ctl_other[a.ctl_slots * kChainCtlStride + i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // the entries of this workgroup: [qb, qe) of the work list; one queue: claimed one by one from all of it
  const bool claiming = a.n_queues == 1u;
  uint32_t qb = 0u, qe = a.q_end;
  if (!claiming) {
    const uint32_t xcc = (uint32_t)__builtin_amdgcn_s_getreg(0x1814) & 15u;       // XCC_ID
    if (xcc >= a.n_queues) {
      // an XCD this launch was not planned for: its workgroups must not touch any entry (completion flags are only
      // valid inside one XCD); the pass is reported as abandoned
      if (tid == 0) __hip_atomic_store(&a.ctl[kChainCtlAbort * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
    if (tid == 0) {
      // shader engine, shader array and compute unit of HW_ID: one of kChainRankWords / kNumXCDs keys per XCD
      const uint32_t cu = ((uint32_t)__builtin_amdgcn_s_getreg(0xF804) >> 8) & 255u;
      const uint32_t arrived = __hip_atomic_fetch_add(&a.ctl[a.ctl_slots * kChainCtlStride + xcc * 256u + cu], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t cls = arrived != 0u ? 1u : 0u;
      const uint32_t drawn = __hip_atomic_fetch_add(&a.ctl[(kChainCtlHead + 2u * xcc + cls) * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_msg[0] = drawn < (uint32_t)kChainColumns ? xcc * 2u * kChainColumns + cls * kChainColumns + drawn : 0xffffffffu;
    }
    __syncthreads();
    const uint32_t col = __builtin_amdgcn_readfirstlane(s_msg[0]);
    __syncthreads();
    if (col == 0xffffffffu) return;        // every column of this kind has its workgroup
    const __attribute__((address_space(4))) uint32_t* cb = (const __attribute__((address_space(4))) uint32_t*)(a.colbegin + col);
    qb = cb[0];
    qe = cb[1];
  }
  uint32_t n_done = 0u;
  {
    uint32_t next = 0xffffffffu;            // one queue, thread 0: the entry claimed ahead
    if (claiming && tid == 0) next = chain_claim(a, 0u, qb, qe);
    for (uint32_t round = 0; round <= qe - qb; ++round) {
      uint32_t idx = qb + round;
      if (claiming) {
        if (tid == 0) s_msg[0] = next;
        __syncthreads();
        idx = __builtin_amdgcn_readfirstlane(s_msg[0]);
      }
      if (idx >= qe) break;
      ConstItem* ip = (ConstItem*)(a.items + idx);
      st_work_item it;
      it.tenant = ip->tenant;
      it.k_split_idx = ip->k_split_idx;
      it.tile_m = ip->tile_m;
      it.tile_n = ip->tile_n;
      it.reserved = 0u;
      ConstOp& T = *(ConstOp*)(a.ops + it.tenant);
      uint64_t* prof = a.prof ? a.prof + (size_t)idx * kProfSlots : nullptr;
      uint64_t waited = 0;
      // one word of every 64-byte line of the op record, requested before the dependency wait and used after it, so
      // that the record sits in the scalar cache when the tile code reads its fields
      const uint32_t rec_touch = (uint32_t)(uintptr_t)T.x ^ (uint32_t)T.R ^ (uint32_t)T.tiles_m ^ T.x_bytes ^ T.chain_flag_base;
      if (T.chain_need != 0u) {
        // Wavefront 0 looks at the dependency: with flags, at those of the sequence's previous stage, 64 at a time from
        // the first that was not yet set (they were stored by workgroups of this XCD and sit, newer than memory, in
        // its L2, where a device-scope load finds them; such a load never stops at the vector cache); with a
        // counter, at the sequence's count of finished entries (bumped by device-scope atomics, carried out at the
        // memory side; a workgroup-scope load would stop at the vector cache and never see it move).
        const bool by_flags = (a.flags & kChainFlagLocalFlags) != 0u;
        const uint32_t* f = a.item_flags + T.chain_dep_begin;
        const uint32_t n = T.chain_dep_count, run = a.run_number, need = T.chain_need;
        const uint32_t* ctr = a.ctl + (kChainCtlSeq + T.chain_seq) * kChainCtlStride;
        uint32_t c0 = 0u;                     // flags before c0 are known to be set
        auto satisfied = [&]() -> bool {      // wavefront 0 only, uniform
          if (!by_flags) return (int32_t)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - need) >= 0;
          while (c0 < n) {
            const uint32_t c = c0 + (uint32_t)tid;
            const bool unset = (c < n) && __hip_atomic_load(f + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != run;
            if (__builtin_amdgcn_ballot_w64(unset) != 0ull) return false;
            c0 += 64u;
          }
          return true;
        };
        // first looks: an entry whose dependency is complete, or completes within a couple of microseconds (the
        // workgroups of a stage finish within about one of each other), starts at once
        if (tid < 64) {
          bool ready = satisfied();
          for (int g = 0; g < kChainGraceLooks && !ready; ++g) {
            __builtin_amdgcn_s_sleep(2);
            ready = satisfied();
          }
          if (tid == 0) s_msg[1] = ready ? 1u : 2u;
        }
        __syncthreads();
        const uint32_t first = s_msg[1];
        if (first == 2u) {
          __syncthreads();                    // s_msg[1] has been read by everyone
          // a longer wait: pull the filter slab closer meanwhile (the touches must have returned before the entry
          // starts, which is why an entry that is about to become ready does not issue them)
          const uint32_t touched = prefetch_filters(T, it, tid);
          if (tid < 64) {
            const uint64_t t0 = wall_clock64();
            uint32_t ok = 1u, polls = 0u;
            while (!satisfied()) {
              // the abort flag and the clock are looked at on every 16th poll (every few microseconds)
              if ((++polls & 15u) != 0u) { __builtin_amdgcn_s_sleep(2); continue; }
              if (__hip_atomic_load(&a.ctl[kChainCtlAbort * kChainCtlStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) { ok = 0u; break; }
              if (wall_clock64() - t0 > (uint64_t)a.spin_limit || polls > kChainMaxPolls) {
                if (tid == 0) __hip_atomic_store(&a.ctl[kChainCtlAbort * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0u;
                break;
              }
              __builtin_amdgcn_s_sleep(2);
            }
            waited = wall_clock64() - t0;
            if (tid == 0) s_msg[1] = ok;
          }
          // No cache is invalidated here: everything an entry reads that this launch wrote (activations, residuals,
          // split-K partial tiles) is read with device-scope loads, and everything else did not change.
          __syncthreads();
          asm volatile("" ::"v"(touched));      // the prefetch loads are complete (and not optimised away)
          if (s_msg[1] == 0u) break;
        }
      }
      asm volatile("" ::"s"(rec_touch));
      if (T.cfg == kChainPoolCfg && prof && tid == 0) prof[4] = wall_clock64();
      chain_item(T, it, smem, prof);
      // Completion.  Outputs were stored write-through; channel counts that are not a multiple of 8 take an epilogue
      // with plain stores and need the release fence (write-back of the L2).
      if (T.cfg != kChainPoolCfg && (T.K & 7) != 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __builtin_amdgcn_s_waitcnt(0);          // every store of this thread has been acknowledged
      __syncthreads();                        // ... of every thread; also: smem and s_msg are free again
      ++n_done;
      if (tid == 0) {
        if ((a.flags & kChainFlagLocalFlags) != 0u) {
          const uint32_t pos = ((uint32_t)it.tile_m * (uint32_t)T.tiles_n + (uint32_t)it.tile_n) * (uint32_t)T.split_k + (uint32_t)it.k_split_idx;
          __hip_atomic_store(a.item_flags + T.chain_flag_base + pos, a.run_number, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        } else {
          __hip_atomic_fetch_add(a.ctl + (kChainCtlSeq + T.chain_seq) * kChainCtlStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // One queue: the following entry is claimed only now.  The claim is a round trip to memory: issued before the
        // entry's work it sits in front of the first operand loads in the in-order memory counter; issued before the
        // completion signal (even as early as the end of the K loop: measured) it delays every dependant.
        if (claiming) next = chain_claim(a, 0u, qb, qe);
        if (prof) {
          prof[7] = waited;
          if (T.cfg == kChainPoolCfg) prof[6] = wall_clock64();
        }
      }
    }
  }
  if (tid == 0 && n_done != 0u) __hip_atomic_fetch_add(&a.ctl[kChainCtlDone * kChainCtlStride], n_done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

int chain_max_workgroups(int* out_workgroups, int* out_xcds) {
  int dev = 0, per_cu = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return (int)e;
  e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, st_chain_kernel, kThreads, 0);
  if (e != hipSuccess) return (int)e;
  if (per_cu < 1) per_cu = 1;
  *out_workgroups = per_cu * prop.multiProcessorCount;
  // an XCD has 32 compute units; a whole MI355X shows 256 of them (8 XCDs), a partition of it fewer
  *out_xcds = prop.multiProcessorCount / (kNumCUs / kNumXCDs);
  return 0;
}

int launch_chain(const TenantDev* ops_dev, const st_work_item* items_dev, uint32_t n_items, const uint32_t* colbegin_dev, uint32_t n_queues,
                 uint32_t* ctl, uint32_t* ctl_other, uint32_t ctl_slots, uint32_t* item_flags, uint32_t run_number,
                 uint32_t spin_limit_ticks, uint32_t flags, int grid, void* stream, uint64_t* prof_dev) {
  if (n_queues != 1u && n_queues != (uint32_t)kNumXCDs) return (int)hipErrorInvalidValue;
  if (grid <= 0 || n_items == 0u) return 0;
  if (((flags & kChainFlagLocalFlags) != 0u) != (n_queues > 1u)) return (int)hipErrorInvalidValue;
  if (n_queues > 1u && (item_flags == nullptr || run_number == 0u || colbegin_dev == nullptr)) return (int)hipErrorInvalidValue;
  ChainArgs a;
  a.ops = ops_dev;
  a.items = items_dev;
  a.ctl = ctl;
  a.ctl_other = ctl_other;
  a.prof = prof_dev;
  a.item_flags = item_flags;
  a.run_number = run_number;
  a.ctl_slots = ctl_slots;
  a.spin_limit = spin_limit_ticks;
  a.flags = flags;
  a.n_queues = n_queues;
  a.q_end = n_items;
  a.colbegin = colbegin_dev;
  hipLaunchKernelGGL(st_chain_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace st
