// Host side of the chain (st_chain_*): validation, per-stage planning through st_conv_plan, the queue, the dependency
// thresholds, the device arena and the persistent launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <new>
#include <vector>

#include "st_host.h"
#include "st_internal.h"

using namespace st;

struct st_chain {
  std::vector<st_chain_op> ops;
  std::vector<st_chain_op_info> info;        // per op, caller's order
  std::vector<TenantDev> table;              // per op, caller's order (host mirror of the device table)
  std::vector<st_work_item> items;           // the queue; item.tenant = op index
  int n_sequences = 0, n_stages = 0;
  bool host_only = false;
  int64_t flops = 0, bytes = 0, workspace_bytes = 0;
  uint32_t ctl_slots = 0;                    // slots of one control block (kChainCtlStride words each)
  uint32_t spin_limit_ticks = 10000000u;     // 100 ms of the 100 MHz constant clock
  uint32_t flags = 0;
  int n_queues = 1;                          // 1, or kNumXCDs
  // one queue: all of items.  Queues per XCD: column j of XCD x is items[colbegin[x * 2 * kChainColumns + j] ..
  // colbegin[.. + j + 1]), the kChainColumns exclusive columns first, then the shared ones
  std::vector<uint32_t> colbegin;
  uint32_t* d_colbegin = nullptr;
  int workgroups = 0;                        // planned size of the launch
  int launch_workgroups = 0;                 // 0 = workgroups; else a smaller size asked for by the caller
  unsigned run_parity = 0;                   // control block the next run uses
  int64_t runs = 0;
  uint32_t run_number = 0;                   // number of the most recent run (per-item completion flags hold it)
  // device
  char* d_arena = nullptr;
  TenantDev* d_ops = nullptr;
  st_work_item* d_items = nullptr;
  uint32_t* d_ctl[2] = {nullptr, nullptr};
  char* d_counters = nullptr;                // split-K arrival counters of all sequences
  size_t counters_bytes = 0;
  uint32_t* d_item_flags = nullptr;          // one completion flag per work item (queue per XCD only)
  size_t item_flags_bytes = 0;
};

static st_status validate_pool(const st_conv_desc& d, int i) {
  if (d.N <= 0 || d.C <= 0 || d.H <= 0 || d.W <= 0 || d.R <= 0 || d.stride <= 0 || d.pad < 0)
    return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): sizes must be positive, pad >= 0", i);
  if (d.R != d.S || d.K != d.C) return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): needs R == S (the window) and K == C", i);
  if (d.pad >= d.R) return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): pad must be smaller than the window", i);
  if (d.H + 2 * (int64_t)d.pad < d.R || d.W + 2 * (int64_t)d.pad < d.R)
    return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): window larger than the padded image", i);
  if (d.in_dtype != ST_DT_F32 && d.in_dtype != ST_DT_BF16 && d.in_dtype != ST_DT_F16)
    return fail(ST_ERR_UNSUPPORTED, "op %d (max-pool): unknown dtype", i);
  if (d.out_dtype != d.in_dtype) return fail(ST_ERR_UNSUPPORTED, "op %d (max-pool): out_dtype must equal in_dtype", i);
  if (d.layout != ST_LAYOUT_NHWC_KRSC) return fail(ST_ERR_UNSUPPORTED, "op %d (max-pool): tensors must be NHWC", i);
  if (d.C % (16 / elem_size(d.in_dtype)) != 0)
    return fail(ST_ERR_UNSUPPORTED, "op %d (max-pool): C must be a multiple of %d", i, 16 / elem_size(d.in_dtype));
  if (!d.x || !d.y || d.x == d.y) return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): x and y must be non-NULL and distinct", i);
  if (d.epilogue != 0 || d.reserved != 0) return fail(ST_ERR_INVALID_ARG, "op %d (max-pool): epilogue and reserved must be 0", i);
  const int64_t P = (d.H + 2 * (int64_t)d.pad - d.R) / d.stride + 1, Q = (d.W + 2 * (int64_t)d.pad - d.R) / d.stride + 1;
  const int64_t es = elem_size(d.in_dtype);
  if ((int64_t)d.N * d.H * d.W * d.C * es >= ((int64_t)1 << 31) || (int64_t)d.N * P * Q * d.C * es >= ((int64_t)1 << 31))
    return fail(ST_ERR_UNSUPPORTED, "op %d (max-pool): tensors must stay below 2^31 bytes", i);
  return ST_OK;
}

static void destroy_chain(st_chain* c) {
  if (!c) return;
  if (c->d_arena) (void)hipFree(c->d_arena);
  delete c;
}

extern "C" st_status st_chain_plan(const st_chain_op* ops, int32_t n_ops, const st_plan_opts* opts, st_chain** out_chain) {
  if (!out_chain) return fail(ST_ERR_INVALID_ARG, "out_chain is NULL");
  *out_chain = nullptr;
  if (n_ops < 0 || (n_ops > 0 && !ops)) return fail(ST_ERR_INVALID_ARG, "ops is NULL or n_ops negative");
  if (n_ops > 65535) return fail(ST_ERR_UNSUPPORTED, "at most 65535 ops per chain");
  st_plan_opts o;
  std::memset(&o, 0, sizeof(o));
  if (opts) o = *opts;
  const bool host_only = o.host_only != 0;
  const int want_queues = o.chain_queues;
  if (want_queues < 0 || want_queues > 2) return fail(ST_ERR_INVALID_ARG, "opts.chain_queues must be 0, 1 or 2");
  o.host_only = 1;          // the stages are planned on the host; the chain owns the one device arena
  o.order = 0;
  o.chain_queues = 0;
  int max_seq = -1;
  for (int i = 0; i < n_ops; ++i) {
    const st_chain_op& op = ops[i];
    if (op.kind != ST_OP_CONV && op.kind != ST_OP_MAXPOOL) return fail(ST_ERR_INVALID_ARG, "op %d: unknown kind %d", i, op.kind);
    if (op.sequence < 0 || op.sequence >= 4096) return fail(ST_ERR_INVALID_ARG, "op %d: sequence must be in [0, 4096)", i);
    if (op.stage < 0) return fail(ST_ERR_INVALID_ARG, "op %d: stage must be >= 0", i);
    if (op.reserved != 0) return fail(ST_ERR_INVALID_ARG, "op %d: reserved must be 0", i);
    if (op.kind == ST_OP_MAXPOOL) {
      st_status s = validate_pool(op.conv, i);
      if (s != ST_OK) return s;
    }
    max_seq = std::max(max_seq, op.sequence);
  }
  st_chain* c = new (std::nothrow) st_chain();
  if (!c) return fail(ST_ERR_OUT_OF_MEMORY, "host allocation failed");
  st_status status = ST_OK;
  std::vector<st_plan*> stage_plans;
  try {
    c->host_only = host_only;
    c->ops.assign(ops, ops + n_ops);
    c->info.resize(n_ops);
    c->table.resize(n_ops);
    c->n_sequences = max_seq + 1;
    // The work is laid out per XCD when every XCD gets at least one sequence (and the device is a whole 8-XCD one);
    // else there is one queue for the chip.  A host-only chain is laid out for a whole device.
    int max_wg = 2 * kNumCUs, n_xcd = kNumXCDs;
    if (!host_only && n_ops > 0) {
      const hipError_t e = (hipError_t)chain_max_workgroups(&max_wg, &n_xcd);
      if (e != hipSuccess) { delete c; return hip_fail(e, "occupancy query (chain kernel)"); }
    }
    if (want_queues == 2 && n_xcd != kNumXCDs) {
      delete c;
      return fail(ST_ERR_UNSUPPORTED, "the per-XCD layout needs a device with %d XCDs, this one shows %d", kNumXCDs, n_xcd);
    }
    c->n_queues = (want_queues == 2 || (want_queues == 0 && n_xcd == kNumXCDs && c->n_sequences >= kNumXCDs)) ? kNumXCDs : 1;
    // per XCD: producer and consumer of a sequence share that XCD's L2, and completion travels through it
    c->flags = c->n_queues > 1 ? kChainFlagLocalFlags : 0u;
    // The shared columns are only used when a compute unit holds two workgroups (the per-XCD layout exists on a whole
    // device only: kNumCUs compute units, max_wg / kNumCUs workgroups on each).
    const bool two_per_cu = max_wg / kNumCUs >= 2;
    const int n_sub = c->n_queues > 1 ? kNumXCDs * 2 * kChainColumns : 1;      // columns, or the one queue
    std::vector<std::vector<st_work_item>> queues((size_t)n_sub);
    std::map<int, std::vector<int>> by_stage;          // stage -> op indices, caller's order
    for (int i = 0; i < n_ops; ++i) by_stage[ops[i].stage].push_back(i);
    c->n_stages = (int)by_stage.size();
    std::vector<int64_t> done((size_t)c->n_sequences, 0);          // work items of each sequence in earlier stages
    // completion flags: one per work item; a sequence's items of one stage are contiguous, op after op
    int64_t flag_total = 0;
    std::vector<int64_t> prev_begin((size_t)c->n_sequences, 0), prev_count((size_t)c->n_sequences, 0);
    // split-K workspace of a sequence: the largest need of any of its stages (its stages never overlap in time)
    std::vector<int64_t> seq_ws((size_t)c->n_sequences, 0), seq_ct((size_t)c->n_sequences, 0);
    struct Use { int op; int64_t ws_off, ct_off; };
    std::vector<Use> uses;
    for (auto& kv : by_stage) {
      std::vector<int> conv_ops, pool_ops;
      for (int i : kv.second) (ops[i].kind == ST_OP_CONV ? conv_ops : pool_ops).push_back(i);
      std::vector<st_conv_desc> descs;
      for (int i : conv_ops) descs.push_back(ops[i].conv);
      st_plan* sp = nullptr;
      status = st_conv_plan(descs.data(), (int32_t)descs.size(), &o, &sp);
      if (status != ST_OK) break;
      stage_plans.push_back(sp);
      std::vector<int64_t> stage_items((size_t)c->n_sequences, 0), stage_ws((size_t)c->n_sequences, 0), stage_ct((size_t)c->n_sequences, 0);
      for (size_t j = 0; j < conv_ops.size(); ++j) {
        const int i = conv_ops[j];
        const int q = ops[i].sequence;
        st_chain_op_info& inf = c->info[i];
        std::memset(&inf, 0, sizeof(inf));
        inf.sequence = q; inf.stage = ops[i].stage; inf.kind = ST_OP_CONV;
        inf.need = (uint32_t)done[q];
        inf.tile = sp->info[j];
        inf.item_count = sp->info[j].item_count;
        TenantDev T = sp->tenants[j];
        T.chain_seq = q;
        T.chain_need = (uint32_t)done[q];
        c->table[i] = T;
        if (sp->info[j].split_k > 1) {
          const st_tenant_info& ti = sp->info[j];
          uses.push_back({i, stage_ws[q], stage_ct[q]});
          stage_ws[q] += (int64_t)ti.tiles_m * ti.tiles_n * ti.split_k * ti.MT * ti.NT;
          stage_ct[q] += (int64_t)ti.tiles_m * ti.tiles_n;
        }
        stage_items[q] += sp->info[j].item_count;
        c->flops += sp->info[j].flops;
        c->bytes += sp->info[j].bytes;
      }
      // queue: the stage's convolution items in the fused order (longest first), then its max-pool items
      std::vector<std::vector<st_work_item>> stage_q((size_t)c->n_queues);
      for (const st_work_item& it : sp->items_fused) {
        st_work_item g = it;
        g.tenant = (uint16_t)conv_ops[it.tenant];
        stage_q[(size_t)(ops[g.tenant].sequence % c->n_queues)].push_back(g);
      }
      for (int i : pool_ops) {
        const st_conv_desc& d = ops[i].conv;
        const int q = ops[i].sequence;
        const int es = elem_size(d.in_dtype), vec = 16 / es;
        const int P = (d.H + 2 * d.pad - d.R) / d.stride + 1, Q = (d.W + 2 * d.pad - d.R) / d.stride + 1;
        const int64_t total = (int64_t)d.N * P * Q * (d.C / vec);
        const int64_t n_it = (total + kThreads - 1) / kThreads;
        st_chain_op_info& inf = c->info[i];
        std::memset(&inf, 0, sizeof(inf));
        inf.sequence = q; inf.stage = ops[i].stage; inf.kind = ST_OP_MAXPOOL;
        inf.need = (uint32_t)done[q];
        inf.item_count = n_it;
        inf.tile.P = P; inf.tile.Q = Q;
        TenantDev T;
        std::memset(&T, 0, sizeof(T));
        T.x = d.x; T.y = d.y;
        T.C = d.C; T.H = d.H; T.W = d.W; T.K = d.C; T.R = d.R; T.S = d.R; T.stride = d.stride; T.pad = d.pad;
        T.P = P; T.Q = Q; T.PQ = P * Q; T.M = (int32_t)total;
        T.in_dtype = d.in_dtype; T.out_dtype = d.in_dtype;
        T.cfg = kChainPoolCfg; T.split_k = 1;
        T.tiles_m = (int32_t)n_it; T.tiles_n = 1;
        T.x_bytes = (uint32_t)((int64_t)d.N * d.H * d.W * d.C * es);
        T.y_bytes = (uint32_t)((int64_t)d.N * P * Q * d.C * es);
        T.chain_seq = q;
        T.chain_need = (uint32_t)done[q];
        c->table[i] = T;
        for (int64_t k = 0; k < n_it; ++k) {
          st_work_item g;
          g.tenant = (uint16_t)i; g.k_split_idx = 0; g.tile_m = (uint32_t)k; g.tile_n = 0; g.reserved = 0;
          stage_q[(size_t)(q % c->n_queues)].push_back(g);
        }
        stage_items[q] += n_it;
      }
      // one queue: as is.  Queues per XCD: the stage's entries (longest first) are dealt to the XCD's columns, to the
      // exclusive ones first, to the shared ones only beyond one per compute unit, then round again; so a stage with
      // no more entries than compute units never shares one, and every column is in stage order
      for (int x = 0; x < c->n_queues; ++x) {
        const std::vector<st_work_item>& sq = stage_q[(size_t)x];
        const size_t ncol = two_per_cu ? 2 * (size_t)kChainColumns : (size_t)kChainColumns;
        for (size_t k = 0; k < sq.size(); ++k)
          queues[c->n_queues > 1 ? (size_t)x * 2 * kChainColumns + k % ncol : 0].push_back(sq[k]);
      }
      std::vector<int64_t> cursor((size_t)c->n_sequences, 0), stage_begin((size_t)c->n_sequences, 0);
      for (int q = 0; q < c->n_sequences; ++q) {
        cursor[q] = stage_begin[q] = flag_total;
        flag_total += stage_items[q];
      }
      for (int i : kv.second) {
        const int q = ops[i].sequence;
        TenantDev& T = c->table[i];
        T.chain_flag_base = (uint32_t)cursor[q];
        cursor[q] += c->info[i].item_count;
        T.chain_dep_begin = (uint32_t)prev_begin[q];
        T.chain_dep_count = (uint32_t)prev_count[q];
        T.chain_reserved = 0;
      }
      for (int q = 0; q < c->n_sequences; ++q) {
        if (stage_items[q] > 0) { prev_begin[q] = stage_begin[q]; prev_count[q] = stage_items[q]; }
        done[q] += stage_items[q];
        seq_ws[q] = std::max(seq_ws[q], stage_ws[q]);
        seq_ct[q] = std::max(seq_ct[q], stage_ct[q]);
      }
    }
    if (status == ST_OK) {
      int64_t total_items = 0;
      for (const auto& qv : queues) total_items += (int64_t)qv.size();
      if (total_items >= ((int64_t)1 << 31)) status = fail(ST_ERR_UNSUPPORTED, "more than 2^31 work items");
    }
    if (status == ST_OK) {
      if (c->n_queues > 1) c->colbegin.assign((size_t)n_sub + 1, 0u);
      for (int qi = 0; qi < n_sub; ++qi) {
        if (c->n_queues > 1) c->colbegin[(size_t)qi] = (uint32_t)c->items.size();
        c->items.insert(c->items.end(), queues[(size_t)qi].begin(), queues[(size_t)qi].end());
      }
      if (c->n_queues > 1) c->colbegin[(size_t)n_sub] = (uint32_t)c->items.size();
    }
    if (status == ST_OK) {
      // arena: [op table][queue][control block x2][split-K counters][completion flags][column boundaries][split-K partial tiles]
      auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
      c->ctl_slots = (uint32_t)(kChainCtlSeq + c->n_sequences);
      int64_t ws_total = 0, ct_total = 0;
      std::vector<int64_t> ws_base((size_t)c->n_sequences, 0), ct_base((size_t)c->n_sequences, 0);
      for (int q = 0; q < c->n_sequences; ++q) {
        ws_base[q] = ws_total; ct_base[q] = ct_total;
        ws_total += seq_ws[q]; ct_total += seq_ct[q];
      }
      c->workspace_bytes = ws_total * 4 + ct_total * 4;
      const size_t off_items = up((size_t)n_ops * sizeof(TenantDev));
      const size_t off_ctl = off_items + up(c->items.size() * sizeof(st_work_item));
      const size_t ctl_words = (size_t)c->ctl_slots * kChainCtlStride + kChainRankWords;   // one control block
      const size_t off_ct = off_ctl + up(ctl_words * 4 * 2);
      const size_t off_flags = off_ct + up((size_t)ct_total * 4);
      const size_t off_cols = off_flags + up(c->n_queues > 1 ? c->items.size() * 4 : 0);
      const size_t off_ws = off_cols + up(c->colbegin.size() * 4);
      const size_t total = off_ws + (size_t)ws_total * 4;
      if (!host_only && n_ops > 0) {
        hipError_t e = hipMalloc((void**)&c->d_arena, total);
        if (e != hipSuccess) status = hip_fail(e, "hipMalloc (chain arena)");
        if (status == ST_OK) {
          for (const Use& u : uses) {
            const int q = ops[u.op].sequence;
            c->table[u.op].ws = (float*)(c->d_arena + off_ws) + ws_base[q] + u.ws_off;
            c->table[u.op].counters = (uint32_t*)(c->d_arena + off_ct) + ct_base[q] + u.ct_off;
          }
          std::vector<char> host(off_ws, 0);
          std::memcpy(host.data(), c->table.data(), (size_t)n_ops * sizeof(TenantDev));
          std::memcpy(host.data() + off_items, c->items.data(), c->items.size() * sizeof(st_work_item));
          if (!c->colbegin.empty()) std::memcpy(host.data() + off_cols, c->colbegin.data(), c->colbegin.size() * 4);
          e = hipMemcpy(c->d_arena, host.data(), off_ws, hipMemcpyHostToDevice);
          if (e != hipSuccess) status = hip_fail(e, "hipMemcpy (chain tables)");
          c->d_ops = (TenantDev*)c->d_arena;
          c->d_items = (st_work_item*)(c->d_arena + off_items);
          c->d_ctl[0] = (uint32_t*)(c->d_arena + off_ctl);
          c->d_ctl[1] = c->d_ctl[0] + ctl_words;
          c->d_counters = c->d_arena + off_ct;
          c->counters_bytes = (size_t)ct_total * 4;
          if (c->n_queues > 1) {
            c->d_item_flags = (uint32_t*)(c->d_arena + off_flags);
            c->item_flags_bytes = c->items.size() * 4;
            c->d_colbegin = (uint32_t*)(c->d_arena + off_cols);
          }
        }
      }
      // one queue: no more workgroups than entries; queues per XCD: every resident slot (a workgroup for which no column
      // is left goes home at once)
      c->workgroups = c->n_queues > 1 ? max_wg : (int)std::min<int64_t>((int64_t)c->items.size(), max_wg);
    }
  } catch (const std::bad_alloc&) {
    status = fail(ST_ERR_OUT_OF_MEMORY, "host allocation failed");
  }
  for (st_plan* sp : stage_plans) st_conv_plan_destroy(sp);
  if (status != ST_OK) {
    destroy_chain(c);
    return status;
  }
  *out_chain = c;
  return ST_OK;
}

static st_status chain_launch(st_chain* c, void* stream, uint64_t* prof_dev) {
  if (!c) return fail(ST_ERR_INVALID_ARG, "chain is NULL");
  if (c->host_only) return fail(ST_ERR_UNSUPPORTED, "chain was built host-only and cannot run");
  if (c->items.empty()) return ST_OK;
  const unsigned p = c->run_parity;
  if (++c->run_number == 0u) {
    // the run numbers have wrapped: forget every flag of the old numbering (a fill kernel, so a capture may hold it)
    if (c->d_item_flags) ST_HIP((hipError_t)launch_zero(c->d_item_flags, (int64_t)((c->item_flags_bytes + 15) & ~(size_t)15), stream));
    c->run_number = 1u;
  }
  ST_HIP((hipError_t)launch_chain(c->d_ops, c->d_items, (uint32_t)c->items.size(), c->d_colbegin, (uint32_t)c->n_queues, c->d_ctl[p],
                                  c->d_ctl[p ^ 1u], c->ctl_slots, c->d_item_flags, c->run_number, c->spin_limit_ticks, c->flags,
                                  c->launch_workgroups > 0 ? c->launch_workgroups : c->workgroups, stream, prof_dev));
  c->run_parity = p ^ 1u;
  ++c->runs;
  return ST_OK;
}

extern "C" st_status st_chain_run(st_chain* chain, void* hip_stream) { return chain_launch(chain, hip_stream, nullptr); }

extern "C" st_status st_chain_run_profiled(st_chain* chain, void* hip_stream, uint64_t* stamps, int64_t capacity) {
  if (!chain) return fail(ST_ERR_INVALID_ARG, "chain is NULL");
  const int64_t n = (int64_t)chain->items.size();
  if (!stamps || capacity < n * kProfSlots) return fail(ST_ERR_INVALID_ARG, "stamps buffer too small: need %lld entries", (long long)(n * kProfSlots));
  if (chain->host_only) return fail(ST_ERR_UNSUPPORTED, "chain was built host-only and cannot run");
  if (n == 0) return ST_OK;
  uint64_t* d = nullptr;
  ST_HIP(hipMalloc((void**)&d, (size_t)n * kProfSlots * 8));
  hipError_t e = (hipError_t)launch_zero(d, n * kProfSlots * 8, hip_stream);
  st_status s = ST_OK;
  if (e == hipSuccess) s = chain_launch(chain, hip_stream, d);
  if (e == hipSuccess && s == ST_OK) e = hipStreamSynchronize((hipStream_t)hip_stream);
  if (e == hipSuccess && s == ST_OK) e = hipMemcpy(stamps, d, (size_t)n * kProfSlots * 8, hipMemcpyDeviceToHost);
  (void)hipFree(d);
  if (s != ST_OK) return s;
  if (e != hipSuccess) return hip_fail(e, "st_chain_run_profiled");
  return ST_OK;
}

extern "C" st_status st_chain_aborted(st_chain* chain, int32_t* aborted) {
  if (!chain || !aborted) return fail(ST_ERR_INVALID_ARG, "NULL argument");
  *aborted = 0;
  if (chain->host_only || chain->items.empty()) return ST_OK;
  ST_HIP(hipDeviceSynchronize());
  uint32_t flag[2] = {0u, 0u}, done = 0u;
  for (int b = 0; b < 2; ++b) ST_HIP(hipMemcpy(&flag[b], chain->d_ctl[b] + kChainCtlAbort * kChainCtlStride, 4, hipMemcpyDeviceToHost));
  // the block of the most recent run still holds its count of completed work items (the other one was cleared by it)
  const unsigned last = chain->run_parity ^ 1u;
  ST_HIP(hipMemcpy(&done, chain->d_ctl[last] + kChainCtlDone * kChainCtlStride, 4, hipMemcpyDeviceToHost));
  const bool incomplete = chain->runs > 0 && done != (uint32_t)chain->items.size();
  if (flag[0] | flag[1] | (incomplete ? 1u : 0u)) {
    // an abandoned pass has left its queue head, its sequence counters and some split-K arrival counters anywhere
    ST_HIP(hipMemset(chain->d_ctl[0], 0, ((size_t)chain->ctl_slots * kChainCtlStride + kChainRankWords) * 4 * 2));
    if (chain->counters_bytes) ST_HIP(hipMemset(chain->d_counters, 0, chain->counters_bytes));
    chain->runs = 0;
    *aborted = 1;
  }
  return ST_OK;
}

extern "C" st_status st_chain_set_wait_limit_us(st_chain* chain, int64_t microseconds) {
  if (!chain) return fail(ST_ERR_INVALID_ARG, "chain is NULL");
  if (microseconds < 0 || microseconds > 40000000) return fail(ST_ERR_INVALID_ARG, "limit must be between 0 and 40 s");
  chain->spin_limit_ticks = (uint32_t)(microseconds * 100);
  return ST_OK;
}

extern "C" st_status st_chain_set_workgroups(st_chain* chain, int32_t workgroups) {
  if (!chain) return fail(ST_ERR_INVALID_ARG, "chain is NULL");
  if (workgroups < 0 || workgroups > chain->workgroups) return fail(ST_ERR_INVALID_ARG, "workgroups must be between 0 and %d", chain->workgroups);
  chain->launch_workgroups = workgroups;
  return ST_OK;
}

extern "C" st_status st_chain_get_info(const st_chain* chain, st_chain_info* out) {
  if (!chain || !out) return fail(ST_ERR_INVALID_ARG, "NULL argument");
  std::memset(out, 0, sizeof(*out));
  out->n_ops = (int32_t)chain->ops.size();
  out->n_sequences = chain->n_sequences;
  out->n_stages = chain->n_stages;
  out->workgroups = chain->workgroups;
  out->n_items = (int64_t)chain->items.size();
  out->flops = chain->flops;
  out->bytes = chain->bytes;
  out->workspace_bytes = chain->workspace_bytes;
  out->host_only = chain->host_only ? 1 : 0;
  out->n_queues = chain->n_queues;
  const int64_t n = (int64_t)chain->items.size();
  for (int q = 0; q <= kNumXCDs; ++q)
    out->queue_begin[q] = chain->n_queues > 1 ? chain->colbegin[(size_t)q * 2 * kChainColumns] : (q == 0 ? 0 : n);
  for (int q = 0; q < kNumXCDs; ++q)
    out->shared_begin[q] = chain->n_queues > 1 ? chain->colbegin[(size_t)q * 2 * kChainColumns + kChainColumns] : out->queue_begin[q + 1];
  out->columns = chain->n_queues > 1 ? kChainColumns : 0;
  return ST_OK;
}

extern "C" st_status st_chain_get_op_info(const st_chain* chain, int32_t op, st_chain_op_info* out) {
  if (!chain || !out) return fail(ST_ERR_INVALID_ARG, "NULL argument");
  if (op < 0 || (size_t)op >= chain->info.size()) return fail(ST_ERR_INVALID_ARG, "op index out of range");
  *out = chain->info[op];
  return ST_OK;
}

extern "C" st_status st_chain_worklist(const st_chain* chain, const st_work_item** items, int64_t* n_items) {
  if (!chain || !items || !n_items) return fail(ST_ERR_INVALID_ARG, "NULL argument");
  *items = chain->items.data();
  *n_items = (int64_t)chain->items.size();
  return ST_OK;
}

extern "C" st_status st_chain_columns(const st_chain* chain, const uint32_t** begins, int64_t* n) {
  if (!chain || !begins || !n) return fail(ST_ERR_INVALID_ARG, "NULL argument");
  *begins = chain->colbegin.empty() ? nullptr : chain->colbegin.data();
  *n = (int64_t)chain->colbegin.size();
  return ST_OK;
}

extern "C" void st_chain_destroy(st_chain* chain) { destroy_chain(chain); }
