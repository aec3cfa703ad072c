/*
 * st_conv.h - C ABI of the fused multi-tenant convolution library for MI355X (gfx950).
 *
 * The problem follows the paper's kernel-level experiment (Section 4.1): a set of independent
 * per-tenant layer problems, each with its own weights and inputs, with all data already resident on
 * the device, is executed under one of three issue policies (Figure 6):
 *   space-time : every tenant's problem in ONE launch whose workgroups are divided among tenants
 *                (the "super-kernel" of Section 4),
 *   time-only  : one launch per tenant, one after another,
 *   space-only : one launch per tenant, each on its own stream.
 * The paper batches same-shape matrix products through a vendor call and names variable-size batching
 * as the route to different shapes (Section 4.1, last paragraph); here each problem is a convolution
 * in implicit im2col form (M = N*P*Q output pixels, Ngemm = K filters, Kgemm = C*R*S, the reading
 * fixed by the worked example of Section 4.1) and shapes may differ per tenant.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers, allocated and owned by the caller, borrowed by the plan
 *     until it is destroyed or the tenant is rebound.  The library never frees them.
 *   - Layout: activations NHWC, weights KRSC (filter-major, channel fastest), outputs NHWC (N,P,Q,K).
 *   - Streams are hipStream_t passed as void*; NULL is the default stream.  Run calls are
 *     asynchronous, never synchronise and never allocate device memory.
 *   - Every function returns st_status; on failure no output argument is written (plan pointers are
 *     left NULL) and st_last_error_message() holds a thread-local description.
 *   - Same plan + same inputs => bitwise identical outputs on every run and under every issue policy
 *     (no floating-point atomics; split-K partials are summed in a fixed order).
 *   - A plan that uses split-K owns a workspace: two runs of the same plan must not overlap in time.
 */
#ifndef ST_CONV_H
#define ST_CONV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ST_OK = 0,
  ST_ERR_INVALID_ARG = 1,   /* NULL pointer, non-positive size, empty output, aliasing, bad index   */
  ST_ERR_UNSUPPORTED = 2,   /* unknown dtype/layout, tensor of 2^31 bytes or more, host-only plan run  */
  ST_ERR_OUT_OF_MEMORY = 3, /* host or device allocation failed                                      */
  ST_ERR_DEVICE = 4         /* any other HIP error (text in st_last_error_message)                   */
} st_status;

typedef enum { ST_DT_F32 = 0, ST_DT_BF16 = 1, ST_DT_F16 = 2 } st_dtype;
/* Only ST_LAYOUT_NHWC_KRSC is implemented: the reduction index is then channel-fastest and contiguous in both
 * operands.  ST_LAYOUT_NCHW_KCRS is named so that callers can ask for it and get ST_ERR_UNSUPPORTED. */
typedef enum { ST_LAYOUT_NHWC_KRSC = 0, ST_LAYOUT_NCHW_KCRS = 1 } st_layout;
enum { ST_EPI_RELU = 1u, ST_EPI_RESIDUAL = 2u };

/* One tenant's layer.  y[n,p,q,k] = sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c]
 * with zeros outside the image, P = floor((H+2*pad-R)/stride)+1 (Q likewise), no bias, dilation 1,
 * groups 1; products are exact in fp32 and accumulated in fp32.  Epilogue order: + residual (read as
 * out_dtype, added in fp32), then ReLU, then rounding to out_dtype (nearest, ties to even). */
typedef struct st_conv_desc {
  int32_t N, C, H, W;    /* input batch, channels, height, width                         */
  int32_t K, R, S;       /* filters, filter height, filter width                         */
  int32_t stride, pad;   /* same in both spatial dimensions                              */
  int32_t in_dtype;      /* st_dtype of x and w                                          */
  int32_t out_dtype;     /* ST_DT_F32 or equal to in_dtype                               */
  int32_t layout;        /* st_layout                                                    */
  uint32_t epilogue;     /* ST_EPI_* bits                                                */
  int32_t reserved;      /* must be 0                                                    */
  const void* x;         /* device, N*H*W*C elements of in_dtype                         */
  const void* w;         /* device, K*R*S*C elements of in_dtype                         */
  void* y;               /* device, N*P*Q*K elements of out_dtype, written               */
  const void* residual;  /* device, same shape and dtype as y; required iff ST_EPI_RESIDUAL */
} st_conv_desc;

/* Planner knobs; pass NULL for defaults.  Zero-initialise, then set what you need. */
typedef struct st_plan_opts {
  int32_t tile_cfg;      /* 0 = choose per tenant; 1 + index into st_tile_shape() to force one       */
  int32_t split_k;       /* 0 = choose per tenant; >= 1 forces that factor (clamped to the K steps)  */
  int32_t order;         /* 0 = longest work item first (default); 1 = tenant-major; 2 = equal        */
                         /* progress: tenants interleaved in proportion to their item counts         */
  int32_t host_only;     /* 1 = build the tables on the host only (no device calls); run => error    */
  int32_t target_items;  /* 0 = default; else the workgroup slots the planner's cost model fills      */
  int32_t rows_per_tile; /* 0 = choose; 1, 2 or 4 forces the output rows per work item of row-tiled   */
                         /* tenants (ignored for the others)                                         */
  int32_t chain_queues;  /* st_chain_plan only: 0 = choose; 1 = one work queue for the whole chip; 2 = the  */
                         /* per-XCD layout, each sequence bound to one XCD (needs a whole 8-XCD device)     */
  int32_t reserved;      /* must be 0                                                                */
} st_plan_opts;

/* One workgroup's assignment: the bit-exact object of the plan.  tile_m counts pixel tiles (MT rows
 * of the im2col matrix), tile_n channel tiles (NT filters), k_split_idx which slice of Kgemm. */
typedef struct st_work_item {
  uint16_t tenant;
  uint16_t k_split_idx;
  uint32_t tile_m;
  uint32_t tile_n;
  uint32_t reserved;
} st_work_item;

typedef struct st_tenant_info {
  int32_t P, Q;
  int64_t M, Ngemm, Kgemm;     /* im2col product sizes                                      */
  int64_t flops;               /* 2*M*Ngemm*Kgemm (padded taps counted)                     */
  int64_t bytes;               /* x + w + y, each element once                              */
  int32_t tile_cfg;            /* index into st_tile_shape()                                */
  int32_t MT, NT;              /* pixels and filters per tile                               */
  int32_t tiles_m, tiles_n;    /* tiles_m = ceil(M/MT), or N*ceil(P/rows_per_tile)*ceil(Q/MT) when row_tiled */
  int32_t split_k;             /* slices of Kgemm per output tile                           */
  int32_t k_steps;             /* K steps (of the tile shape's k_step_bytes per row) over Kgemm */
  int32_t k_steps_per_split;   /* ceil(k_steps / split_k); the last slice may be shorter    */
  int64_t item_begin;          /* slice [item_begin, item_begin+item_count) of the          */
  int64_t item_count;          /*   tenant-major work list belongs to this tenant           */
  int32_t row_tiled;           /* 1: pixel tiles are row segments of consecutive output rows */
  int32_t rows_per_tile;       /* output rows per tile when row_tiled, else 0                */
  int32_t xcd_blocks_m;        /* XCD placement (workgroup b of a launch runs on XCD b mod 8): the tiles are */
  int32_t xcd_blocks_n;        /* cut into xcd_blocks_m ranges of pixel tiles x xcd_blocks_n ranges of filter */
                               /* tiles, at most 8 blocks, each kept on one XCD as far as an even spread allows */
} st_tenant_info;

typedef struct st_plan_info {
  int32_t n_tenants;
  int32_t host_only;
  int64_t n_items;             /* workgroups in the fused launch                            */
  int64_t flops, bytes;        /* sums over tenants                                         */
  int64_t workspace_bytes;     /* split-K partials + counters owned by the plan             */
} st_plan_info;

typedef struct st_plan st_plan; /* opaque */

/* Section 4 (kernels arrive at run time, so super-kernels cannot be built ahead of time): build the
 * launch plan for whatever set of problems is ready.  Validates every descriptor, derives P, Q and the
 * im2col sizes, picks a tile shape and a split-K factor per tenant so that the launch fills the
 * 256 compute units, enumerates the work items, and uploads the tenant table and work lists.
 * n_tenants == 0 gives an empty plan whose runs are no-ops.  Host allocations and (unless
 * opts->host_only) device allocations happen here and only here. */
st_status st_conv_plan(const st_conv_desc* descs, int32_t n_tenants, const st_plan_opts* opts,
                       st_plan** out_plan);

/* Space-time policy (Section 4, Figure 6): one launch, grid = number of work items. */
st_status st_conv_run(const st_plan* plan, void* hip_stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The plan's fused launch (as st_conv_run: same kernel, same work items, bitwise the same
 * outputs) with the tenant table, the work list and the split-K workspace placed in a fixed device array of
 * st_conv_noalloc_max_bytes() = 32 MiB that every GPU the library runs on holds until the process ends, instead
 * of in memory the plan owns.  `plan` may be a host-only plan (st_plan_opts.host_only = 1: built without any
 * device call) or an ordinary one; its tensors are the caller's, as always.  The call allocates no device or
 * pinned memory and calls no copy routine: the tables travel inside the arguments of small launches queued on
 * hip_stream ahead of the convolution launch (about one launch per 3.5 KB of tables), and the arrival counters
 * are cleared by a fill launch.  Asynchronous.  ST_ERR_UNSUPPORTED when tables plus workspace exceed the array
 * (checked before any device call).  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, or several threads) race; calls queued on one stream are ordered by the stream. */
st_status st_conv_run_noalloc(const st_plan* plan, void* hip_stream);
int64_t st_conv_noalloc_max_bytes(void);

/* The fused launch with in-kernel time stamps, for occupancy-per-tenant and latency reports (the
 * per-kernel monitoring Section 4 asks of the scheduler).  Synchronous, allocates a scratch buffer: a
 * diagnostic, not part of the run path.  stamps (HOST pointer) receives 8 uint64 per work item, in
 * fused work-list order: [0] shader-clock at start, [1] first operands staged, [2] K loop done,
 * [3] tile stored (0 for split-K slices that did not do the final reduction), [4] 100 MHz wall clock
 * at start, [5] hardware id (XCC id << 32 | HW_ID register), [6] 100 MHz wall clock at the end,
 * [7] unused. */
st_status st_conv_run_profiled(const st_plan* plan, void* hip_stream, uint64_t* stamps, int64_t capacity);

/* Per-tenant timing of one fused launch (the per-kernel monitoring Section 4 asks of the scheduler; the
 * predictability question of Section 3).  first_start_ns[t] and last_end_ns[t] (HOST arrays of n_tenants
 * entries, n_tenants = the plan's) receive the time from the start of the launch's first workgroup to the
 * start of tenant t's first workgroup and to the end of its last one, from the 100 MHz constant clock
 * (10 ns resolution).  Synchronous diagnostic, like st_conv_run_profiled. */
st_status st_conv_run_tenant_times(const st_plan* plan, void* hip_stream, int64_t* first_start_ns,
                                   int64_t* last_end_ns, int32_t n_tenants);

/* Time-only policy (Section 3, Figure 6): one launch per tenant on one in-order stream, no host
 * synchronisation in between.  Same kernel, same tiles, same work items as st_conv_run. */
st_status st_conv_run_time_only(const st_plan* plan, void* hip_stream);

/* Space-only policy (Section 3 "explicit spatial multiplexing", Figure 6): tenant t is launched on
 * hip_streams[t % n_streams].  hip_streams[0] is the anchor: every other stream first waits for the
 * work already queued on it, and on return it waits for every other stream, so work queued on
 * hip_streams[0] afterwards (e.g. a timing event) follows all tenants.  The first space-only run of a
 * plan creates the events it forks and joins with; later runs create nothing. */
st_status st_conv_run_space_only(const st_plan* plan, void* const* hip_streams, int32_t n_streams);

/* The two baselines with one plan per tenant: every plan is issued as its own launch, serially on one
 * stream (time-only) or plan i on hip_streams[i % n_streams] with the same fork/join convention as
 * st_conv_run_space_only.  Planning each tenant alone lets its tiles and split-K factor suit a launch
 * that has the whole GPU to itself, which is the fairest form of the paper's baselines (Section 4.1
 * used a separately tuned single-problem kernel for them).  Empty (zero-tenant) plans are skipped. */
st_status st_conv_run_plans_time_only(const st_plan* const* plans, int32_t n_plans, void* hip_stream);
st_status st_conv_run_plans_space_only(const st_plan* const* plans, int32_t n_plans, void* const* hip_streams,
                                       int32_t n_streams);

/* plans[i] as one fused launch on hip_streams[i % n_streams], with no ordering between the streams: the
 * free-running form of spatial multiplexing, where each tenant's stream carries its launches back to back and
 * the caller forks and joins the streams when it needs to (once per chain of layers, say, instead of once per
 * layer as st_conv_run_plans_space_only does). */
st_status st_conv_run_plans_on_streams(const st_plan* const* plans, int32_t n_plans, void* const* hip_streams,
                                       int32_t n_streams);
/* The same, `rounds` times over, as a native loop: the free-running baseline of Section 3 with the issue cost of
 * st_pipeline_run_many (from 64 launches on, up to four host threads issue, each owning some of the streams, so the
 * order on every stream is that of the serial loop; the call returns when all launches are issued). */
st_status st_conv_run_plans_on_streams_many(const st_plan* const* plans, int32_t n_plans, void* const* hip_streams,
                                            int32_t n_streams, int32_t rounds);

/* Replace tenant pointers (the cached-plan path of Section 4: same shapes, new inputs).  NULL keeps
 * the current pointer.  Synchronous small upload on the default stream; not for use while a run of
 * this plan is in flight. */
st_status st_conv_plan_rebind(st_plan* plan, int32_t tenant, const void* x, const void* w, void* y,
                              const void* residual);

/* All tenants' pointers at once, from descs[t].x/w/y/residual (everything else in descs is ignored; the
 * plan keeps its shapes).  Nothing happens when no pointer differs from the plan's current ones.
 * Otherwise the device table is updated by one copy ordered on hip_stream, from pinned memory the plan
 * owns: runs queued on that stream before the call still see the old pointers, runs queued after it the
 * new ones.  Runs of this plan on other streams must not overlap the call. */
st_status st_conv_plan_rebind_all(st_plan* plan, const st_conv_desc* descs, int32_t n_tenants, void* hip_stream);

/* Plan cache for dynamically arriving work (Section 4: the scheduler merges whichever kernels are ready,
 * and caches super-kernels so that the cost of scheduling is paid once per distinct merge).  Plans are
 * keyed by the descriptors in order, everything but the four pointers (a NULL and a non-NULL residual
 * differ).  st_plan_cache_get returns the cached plan rebound to the given pointers (as
 * st_conv_plan_rebind_all on hip_stream), or builds one with the cache's options (device allocation,
 * as st_conv_plan) and keeps it; when the cache is full the least recently used plan is destroyed first
 * (which waits for the device).  The returned plan belongs to the cache and stays valid until it is
 * evicted or the cache destroyed.  *out_hit (optional) receives 1 for a cached plan, 0 for a new one.
 * Not thread-safe. */
typedef struct st_plan_cache st_plan_cache;
typedef struct st_plan_cache_stats {
  int64_t hits, misses, evictions;
  int32_t size, capacity;
} st_plan_cache_stats;
st_status st_plan_cache_create(int32_t capacity, const st_plan_opts* opts, st_plan_cache** out_cache);
st_status st_plan_cache_get(st_plan_cache* cache, const st_conv_desc* descs, int32_t n_tenants, void* hip_stream,
                            st_plan** out_plan, int32_t* out_hit);
st_status st_plan_cache_get_stats(const st_plan_cache* cache, st_plan_cache_stats* out);
void st_plan_cache_destroy(st_plan_cache* cache);

/* Several independent batches in flight.  Launches queued on one stream run strictly one after the other, and
 * each pays the drain of the launch before it, the cache write-back and invalidate between them and the start-up
 * of the next (about 3 us here); launches on different streams overlap all of that.  A pipeline is a ring of
 * `depth` streams (default priority, created here, destroyed with it): st_pipeline_next hands out the stream for
 * the next batch, round-robin; the caller queues that batch's launches on it (one st_conv_run, or a whole chain
 * of dependent layers) with tensors no batch still in flight uses.  st_pipeline_slots(depth) is the
 * st_plan_opts.target_items to plan such launches with: when `depth` launches share the GPU, fewer and larger
 * work items beat filling the whole chip once per launch (0 = the planner's default, for depth 1).  This is the
 * space-time trade-off of Section 4 one level up: how much of the GPU one fused launch spans against how many
 * fused launches overlap in time.  st_pipeline_sync waits for every stream of the ring. */
typedef struct st_pipeline st_pipeline;
st_status st_pipeline_create(int32_t depth, st_pipeline** out_pipeline);
int32_t st_pipeline_slots(int32_t depth);
st_status st_pipeline_next(st_pipeline* pipeline, void** out_stream);
/* st_pipeline_next followed by st_conv_run of `plan` on that stream. */
st_status st_pipeline_run(st_pipeline* pipeline, const st_plan* plan);
/* plans[0..n_plans) in order, `rounds` times over, each as st_pipeline_run: a native submission loop (the
 * per-launch cost of a caller in an interpreted language is of the order of the launches themselves).  From 64
 * launches on, the launches are issued by up to four host threads (environment variable ST_PIPELINE_THREADS
 * overrides the count; 1 = the calling thread only), each owning some of the ring's streams, so the order of the
 * launches on every stream is that of the serial loop; the call returns when all are issued.  A launch costs
 * the host about 2.3 us, more than a small fused launch needs once several are in flight. */
st_status st_pipeline_run_many(st_pipeline* pipeline, const st_plan* const* plans, int32_t n_plans, int32_t rounds);
st_status st_pipeline_sync(st_pipeline* pipeline);
void st_pipeline_destroy(st_pipeline* pipeline);

/* ---- A whole chain of dependent layers as ONE launch -------------------------------------------------------
 * The space-time policy of Section 4 applied across layers as well as across tenants: the work items of every
 * op (a convolution layer, or a max-pool) of every tenant go into one queue, and one persistent launch works
 * through it.  Ops are grouped into SEQUENCES (one per tenant network: Section 4's disjoint graphs) and, within a
 * sequence, ordered by STAGE: an op's work items start once every work item of its sequence's ops with a smaller
 * stage is complete; ops of one sequence with equal stage are independent of each other (a block's projection
 * convolution and its first 1x1 convolution, say); different sequences never wait for each other.  The caller
 * guarantees that this order covers every read-after-write, write-after-read and write-after-write between the
 * ops of a sequence, and that sequences share no written tensor.
 *
 * Tiles are chosen per stage (all ops of that stage, over all sequences, planned together as st_conv_plan would).
 * Within a stage the longest work items come first.  There is either one queue for the whole chip, whose entries
 * the resident workgroups claim one by one in stage order, or (the default from 8 sequences on, on a whole 8-XCD
 * device) the work is laid out per XCD, sequence s on XCD s mod 8, served only by the workgroups that run on that
 * XCD: a sequence's activations then stay in one XCD's L2, and a finished work item is announced through that L2 (a
 * flag per work item) instead of through memory.  An XCD's entries are dealt into COLUMNS, each a list of entries in
 * stage order that ONE workgroup works through (it draws its column when it starts; nothing is claimed per entry):
 * 32 "exclusive" columns, drawn by the first workgroup to arrive on each compute unit, and 32 "shared" ones for later
 * arrivals; a stage's entries go to the exclusive columns first and to the shared ones only beyond one per compute
 * unit (two tiles sharing a compute unit each run markedly slower than one that has it to itself).  Activations
 * written during the launch are read with device-scope loads, so no cache is invalidated between stages.
 * The one-queue form completes with any number of resident workgroups; the column form needs a workgroup for every
 * column in use to become resident eventually (on a GPU the launch has to itself all are at once; a caller that shares
 * the GPU with long-running kernels of its own and sees passes abandoned should plan with chain_queues = 1).  Every
 * dependency wait
 * is bounded by a wall-clock limit (default 100 ms) and a poll count, after which the launch abandons the pass:
 * every workgroup leaves, outputs are incomplete, and st_chain_aborted reports it.  Same ops + same inputs =>
 * outputs bitwise identical from run to run, and bitwise identical to running the stages one st_conv_run at a
 * time with the same tiles. */
typedef enum { ST_OP_CONV = 0, ST_OP_MAXPOOL = 1 } st_op_kind;

typedef struct st_chain_op {
  int32_t kind;       /* st_op_kind                                                                       */
  int32_t sequence;   /* 0 <= sequence < 4096                                                             */
  int32_t stage;      /* >= 0; see above                                                                  */
  int32_t reserved;   /* must be 0                                                                        */
  st_conv_desc conv;  /* ST_OP_CONV: the layer.  ST_OP_MAXPOOL: N, C, H, W, R = S = window, stride, pad,  */
                      /* in_dtype = out_dtype, x (N*H*W*C) and y (N*P*Q*C) are used, K must equal C, and   */
                      /* C must be a multiple of the 16-byte vector (8 for 16-bit types, 4 for fp32);     */
                      /* padding never wins the maximum                                                   */
} st_chain_op;

typedef struct st_chain_info {
  int32_t n_ops, n_sequences, n_stages;
  int32_t workgroups;        /* size of the persistent launch (resident workgroup slots, or fewer)    */
  int64_t n_items;           /* queue entries                                                         */
  int64_t flops, bytes;      /* sums over the convolution ops (as st_plan_info)                       */
  int64_t workspace_bytes;   /* split-K partial tiles and counters (shared by a sequence's stages)    */
  int32_t host_only;
  int32_t n_queues;          /* 1, or 8: work laid out per XCD                                        */
  int32_t columns;           /* columns of each kind per XCD (32), or 0 with one queue               */
  int64_t queue_begin[9];    /* XCD (or the one queue) q owns entries [queue_begin[q], queue_begin[q+1]) */
  int64_t shared_begin[8];   /* ... of which [queue_begin[q], shared_begin[q]) are its exclusive columns and  */
                             /* [shared_begin[q], queue_begin[q+1]) its shared ones (empty with one queue)    */
} st_chain_info;

typedef struct st_chain_op_info {
  int32_t sequence, stage, kind;
  uint32_t need;             /* work items of its sequence that must be complete before this op starts */
  int64_t item_count;        /* its work items                                                         */
  st_tenant_info tile;       /* convolution ops: sizes and the planner's choice (item_begin unused)    */
} st_chain_op_info;

typedef struct st_chain st_chain; /* opaque */

/* Validates the ops (as st_conv_plan does; ST_ERR_UNSUPPORTED for a max-pool whose channel count is not a
 * multiple of the vector), plans every stage, builds the queue, allocates and uploads one device arena (tables,
 * queue, control blocks, split-K workspace) unless opts->host_only.  n_ops == 0 gives an empty chain.  opts as for
 * st_conv_plan (order is ignored: the queue order is fixed). */
st_status st_chain_plan(const st_chain_op* ops, int32_t n_ops, const st_plan_opts* opts, st_chain** out_chain);
/* One pass: one launch on hip_stream.  Asynchronous, allocation-free.  Two runs of one chain must not overlap in
 * time (queue them on one stream). */
st_status st_chain_run(st_chain* chain, void* hip_stream);
/* The same with in-kernel time stamps per queue entry (HOST buffer of 8 uint64 per entry, as st_conv_run_profiled;
 * slot [7] = ticks of the 100 MHz clock the entry waited for its dependency).  Synchronous diagnostic. */
st_status st_chain_run_profiled(st_chain* chain, void* hip_stream, uint64_t* stamps, int64_t capacity);
/* Waits for the device, then *aborted = 1 if any run since the last call gave up on a dependency wait, or if the
 * last run did not complete every work item (an XCD that received no workgroups); the chain is reset. */
st_status st_chain_aborted(st_chain* chain, int32_t* aborted);
/* The wall-clock limit of a dependency wait in microseconds (0 = give up at once unless already satisfied: a test
 * hook that makes every kernel still exit normally). */
st_status st_chain_set_wait_limit_us(st_chain* chain, int64_t microseconds);
/* Size of the launch in workgroups (0 = the planned size, st_chain_info.workgroups; at most that).  A test hook
 * too: with fewer workgroups than the column form needs, the undrawn columns' dependants give up after the wait
 * limit and the pass is reported as abandoned, every kernel still exiting normally. */
st_status st_chain_set_workgroups(st_chain* chain, int32_t workgroups);
st_status st_chain_get_info(const st_chain* chain, st_chain_info* out);
st_status st_chain_get_op_info(const st_chain* chain, int32_t op, st_chain_op_info* out);
/* Host copy of the queue, valid until the chain is destroyed; st_work_item.tenant is the op's index in the ops
 * array given to st_chain_plan. */
st_status st_chain_worklist(const st_chain* chain, const st_work_item** items, int64_t* n_items);
/* Host copy of the column boundaries, valid until the chain is destroyed: *n = 8 * 2 * columns + 1 (0 with one
 * queue); column j of XCD x (exclusive: j < columns; shared: columns <= j < 2 * columns) is entries
 * [begins[x * 2 * columns + j], begins[x * 2 * columns + j + 1]) of the work list. */
st_status st_chain_columns(const st_chain* chain, const uint32_t** begins, int64_t* n);
void st_chain_destroy(st_chain* chain);

/* Introspection (used by the bit-exact work-list tests and by reports). */
st_status st_conv_plan_info(const st_plan* plan, st_plan_info* out);
st_status st_conv_plan_tenant_info(const st_plan* plan, int32_t tenant, st_tenant_info* out);
/* Host copies of the work lists, valid until the plan is destroyed.  which: 0 = order used by the
 * fused launch, 1 = tenant-major order used by the two baselines. */
st_status st_conv_plan_worklist(const st_plan* plan, int32_t which, const st_work_item** items,
                                int64_t* n_items);
void st_conv_plan_destroy(st_plan* plan);

/* Tile family: shape of config `index` (pixels x filters) and the bytes of the reduction index it
 * stages per row per K step; returns ST_ERR_INVALID_ARG past the end. */
st_status st_tile_shape(int32_t index, int32_t* MT, int32_t* NT, int32_t* k_step_bytes);
int32_t st_tile_count(void);

/* 3x3 / stride 2 / pad 1 style max-pool on an NHWC tensor, the one non-convolution step between the
 * stem and the first bottleneck of a ResNet-50-shaped stack.  x: N*H*W*C, y: N*P*Q*C elements of
 * `dtype`, device pointers; padding never wins the maximum.  Asynchronous on hip_stream. */
st_status st_maxpool_nhwc(const void* x, void* y, int32_t N, int32_t H, int32_t W, int32_t C,
                          int32_t win, int32_t stride, int32_t pad, int32_t dtype, void* hip_stream);

/* Launches an empty kernel: measures the launch floor the fused policy pays once. */
st_status st_launch_empty(void* hip_stream);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned
 * device memory): a kernel of known traffic against which hardware byte counters are scaled. */
st_status st_launch_copy(const void* src, void* dst, int64_t bytes, void* hip_stream);

const char* st_status_string(st_status s);
const char* st_last_error_message(void);

#ifdef __cplusplus
}
#endif
#endif /* ST_CONV_H */
