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
// Memory: producers write their outputs through to memory (device-scope stores) and wait for them before one
// device-scope atomic bumps the sequence's counter; a consumer that has seen the counter reach its threshold
// invalidates its caches (device-scope acquire) before it loads.
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
  uint32_t ctl_slots;     // slots of a control block (one live word per 256-byte slot)
  uint32_t spin_limit;    // ticks of the 100 MHz constant clock a dependency wait may last
  uint32_t flags;         // kChainFlag*
  uint32_t n_queues;      // 1: one queue for the whole chip; kNumXCDs: queue x is served by the workgroups on XCD x
  uint32_t qbegin[kNumXCDs + 1];   // queue q is items[qbegin[q] .. qbegin[q + 1])
};

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
  const u32x4 v = maxpool_vector<DT>(T.x, idx, T.H, T.W, T.C, T.P, T.Q, T.R, T.stride, T.pad);
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
      case ST_DT_BF16: run_dtype<ST_DT_BF16>(T, it, smem, prof); break;
      case ST_DT_F16: run_dtype<ST_DT_F16>(T, it, smem, prof); break;
      default: run_dtype<ST_DT_F32>(T, it, smem, prof); break;
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

__global__ __launch_bounds__(kThreads, 2) void st_chain_kernel(const ChainArgs a) {
  __shared__ __attribute__((aligned(16))) char smem[kSmemBytes];
  __shared__ uint32_t s_msg[2];
  const int tid = threadIdx.x;
  if (blockIdx.x == 0) {
    // the control block of the NEXT run (runs alternate between two blocks; the stream orders them)
    for (uint32_t i = (uint32_t)tid; i < a.ctl_slots; i += kThreads)
      __hip_atomic_store(&a.ctl_other[i * kChainCtlStride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // which queue this workgroup serves: with one queue per XCD, the one of the XCD it runs on
  uint32_t q = 0u;
  if (a.n_queues > 1u) {
    q = (uint32_t)__builtin_amdgcn_s_getreg(0x1814) & 15u;       // XCC_ID
    if (q >= a.n_queues) {
      // an XCD this launch was not planned for: its workgroups must not touch any queue (the light acquire below is
      // only valid inside one XCD); the pass is reported as abandoned
      if (tid == 0) __hip_atomic_store(&a.ctl[kChainCtlAbort * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
  }
  const uint32_t qb = a.qbegin[q], qe = a.qbegin[q + 1];
  uint32_t next = 0xffffffffu;            // thread 0: the entry claimed ahead
  uint32_t n_done = 0u;
  if (tid == 0) next = chain_claim(a, q, qb, qe);
  for (uint32_t round = 0; round <= qe - qb; ++round) {
    if (tid == 0) s_msg[0] = next;
    __syncthreads();
    const uint32_t idx = __builtin_amdgcn_readfirstlane(s_msg[0]);
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
    if (T.chain_need != 0u) {
      const uint32_t touched = prefetch_filters(T, it, tid);
      if (tid == 0) {
        uint32_t* ctr = a.ctl + (kChainCtlSeq + T.chain_seq) * kChainCtlStride;
        const uint32_t need = T.chain_need;
        const uint64_t t0 = wall_clock64();
        uint32_t ok = 1u, polls = 0u;
        // Device-scope atomics are carried out at the memory side: a load that stops at the XCD's L2 never sees the
        // counter move (measured: such polls time out), so every poll is a device-scope load, a round trip to memory.
        auto poll = [&]() -> uint32_t { return __hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
        while ((int32_t)(poll() - need) < 0) {
          // the abort flag and the clock are looked at on every 16th poll (every few microseconds)
          if ((++polls & 15u) != 0u) { __builtin_amdgcn_s_sleep(4); continue; }
          if (__hip_atomic_load(&a.ctl[kChainCtlAbort * kChainCtlStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) { ok = 0u; break; }
          if (wall_clock64() - t0 > (uint64_t)a.spin_limit || polls > kChainMaxPolls) {
            __hip_atomic_store(&a.ctl[kChainCtlAbort * kChainCtlStride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = 0u;
            break;
          }
          __builtin_amdgcn_s_sleep(4);
        }
        waited = wall_clock64() - t0;
        // What the producers wrote (through, to the L2 and to memory) must not be served from a stale cache.  One
        // queue per XCD: producer and consumer share the XCD's L2, so only this compute unit's vector cache can be
        // stale (the acquire of a workgroup spread over compute units).  One queue for the chip: device-scope acquire.
        if (a.flags & kChainFlagAcquireAgent) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        else if (a.flags & kChainFlagAcquireL1) asm volatile("buffer_inv sc0" ::: "memory");
        s_msg[1] = ok;
      }
      __syncthreads();
      asm volatile("" ::"v"(touched));      // the prefetch loads are complete (and not optimised away)
      if (s_msg[1] == 0u) break;
    }
    if (T.cfg == kChainPoolCfg && prof && tid == 0) prof[4] = wall_clock64();
    chain_item(T, it, smem, prof);
    // The following entry is claimed now: the atomic's round trip then overlaps the wait for this entry's stores.
    // (Claimed before the entry's work it would sit at the head of the in-order memory counter and hold up the
    // entry's first operand loads by its whole round trip.)
    if (tid == 0) next = chain_claim(a, q, qb, qe);
    // Completion.  Outputs were stored write-through; channel counts that are not a multiple of 8 take an epilogue
    // with plain stores and need the full release fence.
    if ((a.flags & kChainFlagReleaseFence) != 0u || (T.cfg != kChainPoolCfg && (T.K & 7) != 0)) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __builtin_amdgcn_s_waitcnt(0);          // every store of this thread has been acknowledged
    __syncthreads();                        // ... of every thread; also: smem and s_msg are free again
    ++n_done;
    if (tid == 0) {
      __hip_atomic_fetch_add(a.ctl + (kChainCtlSeq + T.chain_seq) * kChainCtlStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (prof) {
        prof[7] = waited;
        if (T.cfg == kChainPoolCfg) prof[6] = wall_clock64();
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

int launch_chain(const TenantDev* ops_dev, const st_work_item* items_dev, const uint32_t* qbegin, uint32_t n_queues, uint32_t* ctl,
                 uint32_t* ctl_other, uint32_t ctl_slots, uint32_t spin_limit_ticks, uint32_t flags, int grid, void* stream,
                 uint64_t* prof_dev) {
  if (grid <= 0 || n_queues < 1 || n_queues > (uint32_t)kNumXCDs || qbegin[n_queues] == 0u) return 0;
  ChainArgs a;
  a.ops = ops_dev;
  a.items = items_dev;
  a.ctl = ctl;
  a.ctl_other = ctl_other;
  a.prof = prof_dev;
  a.ctl_slots = ctl_slots;
  a.spin_limit = spin_limit_ticks;
  a.flags = flags;
  a.n_queues = n_queues;
  for (int q = 0; q <= kNumXCDs; ++q) a.qbegin[q] = qbegin[q <= (int)n_queues ? q : (int)n_queues];
  hipLaunchKernelGGL(st_chain_kernel, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace st
