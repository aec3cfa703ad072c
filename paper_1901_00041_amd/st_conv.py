"""Thin ctypes binding of libst_conv.so: same names as the C ABI (include/st_conv.h), argument
marshalling only.  Every step of the path runs in the library's HIP kernels; there is no fallback:
if the shared library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libst_conv.so")

ST_OK, ST_ERR_INVALID_ARG, ST_ERR_UNSUPPORTED, ST_ERR_OUT_OF_MEMORY, ST_ERR_DEVICE = range(5)
ST_DT_F32, ST_DT_BF16, ST_DT_F16 = 0, 1, 2
ST_LAYOUT_NHWC_KRSC, ST_LAYOUT_NCHW_KCRS = 0, 1
ST_EPI_RELU, ST_EPI_RESIDUAL = 1, 2
ST_OP_CONV, ST_OP_MAXPOOL = 0, 1
DTYPE_CODE = {"f32": ST_DT_F32, "bf16": ST_DT_BF16, "f16": ST_DT_F16}

EXPORTS = ["st_conv_plan", "st_conv_run", "st_conv_run_noalloc", "st_conv_noalloc_max_bytes", "st_conv_run_profiled", "st_conv_run_tenant_times", "st_conv_run_time_only", "st_conv_run_space_only",
           "st_conv_run_plans_time_only", "st_conv_run_plans_space_only", "st_conv_run_plans_on_streams", "st_conv_run_plans_on_streams_many", "st_conv_plan_rebind", "st_conv_plan_rebind_all",
           "st_pipeline_create", "st_pipeline_slots", "st_pipeline_next", "st_pipeline_run", "st_pipeline_run_many", "st_pipeline_sync", "st_pipeline_destroy",
           "st_plan_cache_create", "st_plan_cache_get", "st_plan_cache_get_stats", "st_plan_cache_destroy", "st_conv_plan_info", "st_conv_plan_tenant_info", "st_conv_plan_worklist",
           "st_conv_plan_destroy", "st_chain_plan", "st_chain_run", "st_chain_run_profiled", "st_chain_aborted", "st_chain_set_wait_limit_us",
           "st_chain_get_info", "st_chain_get_op_info", "st_chain_worklist", "st_chain_columns", "st_chain_set_workgroups", "st_chain_destroy", "st_tile_shape", "st_tile_count", "st_maxpool_nhwc",
           "st_launch_empty", "st_launch_copy", "st_status_string", "st_last_error_message"]


class st_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad",
                                              "in_dtype", "out_dtype", "layout")] + \
               [("epilogue", ctypes.c_uint32), ("reserved", ctypes.c_int32),
                ("x", ctypes.c_void_p), ("w", ctypes.c_void_p), ("y", ctypes.c_void_p),
                ("residual", ctypes.c_void_p)]


class st_plan_opts(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("tile_cfg", "split_k", "order", "host_only", "target_items",
                                                 "rows_per_tile", "chain_queues", "reserved")]


class st_work_item(ctypes.Structure):
    _fields_ = [("tenant", ctypes.c_uint16), ("k_split_idx", ctypes.c_uint16), ("tile_m", ctypes.c_uint32),
                ("tile_n", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


WORK_ITEM_DTYPE = np.dtype([("tenant", "<u2"), ("k_split_idx", "<u2"), ("tile_m", "<u4"), ("tile_n", "<u4"),
                            ("reserved", "<u4")])


class st_tenant_info(ctypes.Structure):
    _fields_ = [("P", ctypes.c_int32), ("Q", ctypes.c_int32), ("M", ctypes.c_int64), ("Ngemm", ctypes.c_int64),
                ("Kgemm", ctypes.c_int64), ("flops", ctypes.c_int64), ("bytes", ctypes.c_int64),
                ("tile_cfg", ctypes.c_int32), ("MT", ctypes.c_int32), ("NT", ctypes.c_int32),
                ("tiles_m", ctypes.c_int32), ("tiles_n", ctypes.c_int32), ("split_k", ctypes.c_int32),
                ("k_steps", ctypes.c_int32), ("k_steps_per_split", ctypes.c_int32),
                ("item_begin", ctypes.c_int64), ("item_count", ctypes.c_int64),
                ("row_tiled", ctypes.c_int32), ("rows_per_tile", ctypes.c_int32),
                ("xcd_blocks_m", ctypes.c_int32), ("xcd_blocks_n", ctypes.c_int32)]


class st_plan_info(ctypes.Structure):
    _fields_ = [("n_tenants", ctypes.c_int32), ("host_only", ctypes.c_int32), ("n_items", ctypes.c_int64),
                ("flops", ctypes.c_int64), ("bytes", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64)]


class st_chain_op(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("sequence", ctypes.c_int32), ("stage", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("conv", st_conv_desc)]


class st_chain_info(ctypes.Structure):
    _fields_ = [("n_ops", ctypes.c_int32), ("n_sequences", ctypes.c_int32), ("n_stages", ctypes.c_int32),
                ("workgroups", ctypes.c_int32), ("n_items", ctypes.c_int64), ("flops", ctypes.c_int64),
                ("bytes", ctypes.c_int64), ("workspace_bytes", ctypes.c_int64), ("host_only", ctypes.c_int32),
                ("n_queues", ctypes.c_int32), ("columns", ctypes.c_int32), ("queue_begin", ctypes.c_int64 * 9),
                ("shared_begin", ctypes.c_int64 * 8)]


class st_chain_op_info(ctypes.Structure):
    _fields_ = [("sequence", ctypes.c_int32), ("stage", ctypes.c_int32), ("kind", ctypes.c_int32), ("need", ctypes.c_uint32),
                ("item_count", ctypes.c_int64), ("tile", st_tenant_info)]


class st_plan_cache_stats(ctypes.Structure):
    _fields_ = [("hits", ctypes.c_int64), ("misses", ctypes.c_int64), ("evictions", ctypes.c_int64),
                ("size", ctypes.c_int32), ("capacity", ctypes.c_int32)]


class StError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().st_last_error_message().decode()
        super().__init__(f"{where}: {lib().st_status_string(status).decode()}: {msg}")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it was never built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1901_00041_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        P = ctypes.POINTER
        L.st_conv_plan.argtypes = [P(st_conv_desc), i32, P(st_plan_opts), P(vp)]
        L.st_conv_run.argtypes = [vp, vp]
        L.st_conv_run_time_only.argtypes = [vp, vp]
        L.st_conv_run_noalloc.argtypes = [vp, vp]
        L.st_conv_run_noalloc.restype = i32
        L.st_conv_noalloc_max_bytes.argtypes = []
        L.st_conv_noalloc_max_bytes.restype = i64
        L.st_conv_run_profiled.argtypes = [vp, vp, P(ctypes.c_uint64), i64]
        L.st_conv_run_space_only.argtypes = [vp, P(vp), i32]
        L.st_conv_run_tenant_times.argtypes = [vp, vp, P(i64), P(i64), i32]
        L.st_conv_run_tenant_times.restype = i32
        L.st_conv_plan_rebind.argtypes = [vp, i32, vp, vp, vp, vp]
        L.st_conv_plan_rebind_all.argtypes = [vp, P(st_conv_desc), i32, vp]
        L.st_plan_cache_create.argtypes = [i32, P(st_plan_opts), P(vp)]
        L.st_plan_cache_get.argtypes = [vp, P(st_conv_desc), i32, vp, P(vp), P(i32)]
        L.st_plan_cache_get_stats.argtypes = [vp, P(st_plan_cache_stats)]
        L.st_plan_cache_destroy.argtypes = [vp]
        L.st_plan_cache_destroy.restype = None
        L.st_pipeline_create.argtypes = [i32, P(vp)]
        L.st_pipeline_create.restype = i32
        L.st_pipeline_slots.argtypes = [i32]
        L.st_pipeline_slots.restype = i32
        L.st_pipeline_next.argtypes = [vp, P(vp)]
        L.st_pipeline_next.restype = i32
        L.st_pipeline_run.argtypes = [vp, vp]
        L.st_pipeline_run.restype = i32
        L.st_pipeline_run_many.argtypes = [vp, P(vp), i32, i32]
        L.st_pipeline_run_many.restype = i32
        L.st_pipeline_sync.argtypes = [vp]
        L.st_pipeline_sync.restype = i32
        L.st_pipeline_destroy.argtypes = [vp]
        L.st_pipeline_destroy.restype = None
        L.st_conv_run_plans_time_only.argtypes = [P(vp), i32, vp]
        L.st_conv_run_plans_space_only.argtypes = [P(vp), i32, P(vp), i32]
        L.st_conv_run_plans_on_streams.argtypes = [P(vp), i32, P(vp), i32]
        L.st_conv_run_plans_on_streams.restype = i32
        L.st_conv_run_plans_on_streams_many.argtypes = [P(vp), i32, P(vp), i32, i32]
        L.st_conv_run_plans_on_streams_many.restype = i32
        L.st_conv_plan_info.argtypes = [vp, P(st_plan_info)]
        L.st_conv_plan_tenant_info.argtypes = [vp, i32, P(st_tenant_info)]
        L.st_conv_plan_worklist.argtypes = [vp, i32, P(P(st_work_item)), P(i64)]
        L.st_conv_plan_destroy.argtypes = [vp]
        L.st_conv_plan_destroy.restype = None
        L.st_chain_plan.argtypes = [P(st_chain_op), i32, P(st_plan_opts), P(vp)]
        L.st_chain_run.argtypes = [vp, vp]
        L.st_chain_run_profiled.argtypes = [vp, vp, P(ctypes.c_uint64), i64]
        L.st_chain_aborted.argtypes = [vp, P(i32)]
        L.st_chain_set_wait_limit_us.argtypes = [vp, i64]
        L.st_chain_set_workgroups.argtypes = [vp, i32]
        L.st_chain_get_info.argtypes = [vp, P(st_chain_info)]
        L.st_chain_get_op_info.argtypes = [vp, i32, P(st_chain_op_info)]
        L.st_chain_worklist.argtypes = [vp, P(P(st_work_item)), P(i64)]
        L.st_chain_columns.argtypes = [vp, P(P(ctypes.c_uint32)), P(i64)]
        L.st_chain_destroy.argtypes = [vp]
        L.st_chain_destroy.restype = None
        for name in ("st_chain_plan", "st_chain_run", "st_chain_run_profiled", "st_chain_aborted", "st_chain_set_wait_limit_us",
                     "st_chain_get_info", "st_chain_get_op_info", "st_chain_worklist", "st_chain_columns", "st_chain_set_workgroups"):
            getattr(L, name).restype = i32
        L.st_tile_shape.argtypes = [i32, P(i32), P(i32), P(i32)]
        L.st_tile_count.argtypes = []
        L.st_maxpool_nhwc.argtypes = [vp, vp] + [i32] * 8 + [vp]
        L.st_launch_empty.argtypes = [vp]
        L.st_launch_copy.argtypes = [vp, vp, i64, vp]
        L.st_status_string.argtypes = [i32]
        L.st_status_string.restype = ctypes.c_char_p
        L.st_last_error_message.argtypes = []
        L.st_last_error_message.restype = ctypes.c_char_p
        for name in ("st_conv_plan", "st_conv_run", "st_conv_run_profiled", "st_conv_run_plans_time_only",
                     "st_conv_run_plans_space_only", "st_conv_run_time_only", "st_conv_run_space_only",
                     "st_conv_plan_rebind", "st_conv_plan_rebind_all", "st_plan_cache_create", "st_plan_cache_get",
                     "st_plan_cache_get_stats", "st_conv_plan_info", "st_conv_plan_tenant_info",
                     "st_conv_plan_worklist", "st_tile_shape", "st_tile_count",
                     "st_maxpool_nhwc", "st_launch_empty", "st_launch_copy"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor, or an integer address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return int(s.cuda_stream)


def make_desc(N, C, H, W, K, R, S, stride, pad, in_dtype, out_dtype, x, w, y, residual=None,
              epilogue=0, layout=ST_LAYOUT_NHWC_KRSC) -> st_conv_desc:
    d = st_conv_desc()
    d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.pad = N, C, H, W, K, R, S, stride, pad
    d.in_dtype = DTYPE_CODE.get(in_dtype, in_dtype)
    d.out_dtype = DTYPE_CODE.get(out_dtype, out_dtype)
    d.layout, d.epilogue, d.reserved = layout, epilogue, 0
    d.x, d.w, d.y, d.residual = _ptr(x), _ptr(w), _ptr(y), _ptr(residual)
    return d


class Plan:
    """Owns an st_plan*; keeps the tensors it borrows alive."""

    def __init__(self, handle: int, keep):
        self.handle = handle
        self._keep = keep

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "handle", None) and _lib is not None:
            try:
                _lib.st_conv_plan_destroy(self.handle)
            except Exception:      # interpreter shutdown
                pass
            self.handle = None


class BorrowedPlan(Plan):
    """A plan handle owned by someone else (a plan cache): never destroyed from here."""

    def __init__(self, handle: int):
        self.handle = handle
        self._keep = None

    def destroy(self):
        self.handle = None


def st_conv_plan(descs: Sequence[st_conv_desc], opts: Optional[st_plan_opts] = None, keep=None) -> Plan:
    n = len(descs)
    arr = (st_conv_desc * max(n, 1))(*descs)
    out = ctypes.c_void_p()
    st = lib().st_conv_plan(arr, n, ctypes.byref(opts) if opts is not None else None, ctypes.byref(out))
    if st != ST_OK:
        raise StError(st, "st_conv_plan")
    return Plan(out.value, keep)


def plan_opts(tile_cfg=0, split_k=0, order=0, host_only=0, target_items=0, rows_per_tile=0, chain_queues=0) -> st_plan_opts:
    o = st_plan_opts()
    o.tile_cfg, o.split_k, o.order, o.host_only, o.target_items = tile_cfg, split_k, order, host_only, target_items
    o.rows_per_tile, o.chain_queues = rows_per_tile, chain_queues
    return o


def _check(st, where):
    if st != ST_OK:
        raise StError(st, where)


def st_conv_run(plan: Plan, stream=None) -> None:
    _check(lib().st_conv_run(plan.handle, _stream(stream)), "st_conv_run")


def st_conv_run_noalloc(plan: Plan, stream=None) -> None:
    _check(lib().st_conv_run_noalloc(plan.handle, _stream(stream)), "st_conv_run_noalloc")


def st_conv_noalloc_max_bytes() -> int:
    return int(lib().st_conv_noalloc_max_bytes())


def st_conv_run_profiled(plan: Plan, stream=None) -> np.ndarray:
    """Fused launch with time stamps; returns an (n_items, 8) uint64 array (see st_conv.h)."""
    n = int(st_conv_plan_info(plan).n_items)
    out = np.zeros((max(n, 1), 8), dtype=np.uint64)
    _check(lib().st_conv_run_profiled(plan.handle, _stream(stream), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                      out.size), "st_conv_run_profiled")
    return out[:n]


def st_conv_run_tenant_times(plan: Plan, stream=None):
    """One fused launch with per-tenant timing; returns (first_start_ns, last_end_ns) int64 arrays."""
    n = int(st_conv_plan_info(plan).n_tenants)
    a, b = np.zeros(max(n, 1), dtype=np.int64), np.zeros(max(n, 1), dtype=np.int64)
    i64p = ctypes.POINTER(ctypes.c_int64)
    _check(lib().st_conv_run_tenant_times(plan.handle, _stream(stream), a.ctypes.data_as(i64p), b.ctypes.data_as(i64p), n),
           "st_conv_run_tenant_times")
    return a[:n], b[:n]


def st_conv_run_time_only(plan: Plan, stream=None) -> None:
    _check(lib().st_conv_run_time_only(plan.handle, _stream(stream)), "st_conv_run_time_only")


def st_conv_run_space_only(plan: Plan, streams) -> None:
    hs = [_stream(s) for s in streams]
    arr = (ctypes.c_void_p * max(len(hs), 1))(*hs)
    _check(lib().st_conv_run_space_only(plan.handle, arr, len(hs)), "st_conv_run_space_only")


def _plan_array(plans):
    return (ctypes.c_void_p * max(len(plans), 1))(*[p.handle for p in plans])


def st_conv_run_plans_time_only(plans, stream=None) -> None:
    _check(lib().st_conv_run_plans_time_only(_plan_array(plans), len(plans), _stream(stream)), "st_conv_run_plans_time_only")


def st_conv_run_plans_space_only(plans, streams) -> None:
    hs = [_stream(s) for s in streams]
    arr = (ctypes.c_void_p * max(len(hs), 1))(*hs)
    _check(lib().st_conv_run_plans_space_only(_plan_array(plans), len(plans), arr, len(hs)), "st_conv_run_plans_space_only")


def st_conv_run_plans_on_streams(plans, streams) -> None:
    hs = [_stream(s) for s in streams]
    arr = (ctypes.c_void_p * max(len(hs), 1))(*hs)
    _check(lib().st_conv_run_plans_on_streams(_plan_array(plans), len(plans), arr, len(hs)), "st_conv_run_plans_on_streams")


def st_conv_run_plans_on_streams_many(plans, streams, rounds: int) -> None:
    hs = [_stream(s) for s in streams]
    arr = (ctypes.c_void_p * max(len(hs), 1))(*hs)
    _check(lib().st_conv_run_plans_on_streams_many(_plan_array(plans), len(plans), arr, len(hs), rounds),
           "st_conv_run_plans_on_streams_many")


def st_conv_plan_rebind(plan: Plan, tenant: int, x=None, w=None, y=None, residual=None) -> None:
    _check(lib().st_conv_plan_rebind(plan.handle, tenant, _ptr(x), _ptr(w), _ptr(y), _ptr(residual)),
           "st_conv_plan_rebind")
    if plan._keep is not None:
        plan._keep.append((x, w, y, residual))


def st_conv_plan_rebind_all(plan: Plan, descs: Sequence[st_conv_desc], stream=None, keep=None) -> None:
    n = len(descs)
    arr = (st_conv_desc * max(n, 1))(*descs)
    _check(lib().st_conv_plan_rebind_all(plan.handle, arr, n, _stream(stream)), "st_conv_plan_rebind_all")
    if keep is not None and plan._keep is not None:
        plan._keep.append(keep)


class Pipeline:
    """Owns an st_pipeline*: a ring of streams for several independent batches in flight."""

    def __init__(self, depth: int):
        out = ctypes.c_void_p()
        _check(lib().st_pipeline_create(depth, ctypes.byref(out)), "st_pipeline_create")
        self.handle, self.depth = out.value, depth
        self.slots = int(lib().st_pipeline_slots(depth))      # st_plan_opts.target_items for launches queued here

    def next(self) -> int:
        """Raw hipStream_t (as an integer) for the next batch."""
        out = ctypes.c_void_p()
        _check(lib().st_pipeline_next(self.handle, ctypes.byref(out)), "st_pipeline_next")
        return int(out.value)

    def run(self, plan) -> None:
        """The plan's fused launch on the next stream of the ring."""
        _check(lib().st_pipeline_run(self.handle, plan.handle), "st_pipeline_run")

    def run_many(self, plans, rounds: int = 1) -> None:
        """plans in order, `rounds` times over, each on the next stream of the ring (one native loop)."""
        _check(lib().st_pipeline_run_many(self.handle, _plan_array(plans), len(plans), rounds), "st_pipeline_run_many")

    def sync(self) -> None:
        _check(lib().st_pipeline_sync(self.handle), "st_pipeline_sync")

    def destroy(self):
        if getattr(self, "handle", None) and _lib is not None:
            try:
                _lib.st_pipeline_destroy(self.handle)
            except Exception:      # interpreter shutdown
                pass
            self.handle = None

    def __del__(self):
        self.destroy()


class PlanCache:
    """Owns an st_plan_cache*.  Plans returned by get() belong to the cache: they are plain handles wrapped
    without ownership, valid until evicted or until the cache is destroyed."""

    def __init__(self, capacity: int, opts: Optional[st_plan_opts] = None):
        out = ctypes.c_void_p()
        _check(lib().st_plan_cache_create(capacity, ctypes.byref(opts) if opts is not None else None, ctypes.byref(out)),
               "st_plan_cache_create")
        self.handle = out.value

    def get(self, descs: Sequence[st_conv_desc], stream=None):
        """Returns (plan, hit)."""
        n = len(descs)
        arr = (st_conv_desc * max(n, 1))(*descs)
        out, hit = ctypes.c_void_p(), ctypes.c_int32()
        _check(lib().st_plan_cache_get(self.handle, arr, n, _stream(stream), ctypes.byref(out), ctypes.byref(hit)),
               "st_plan_cache_get")
        return BorrowedPlan(out.value), bool(hit.value)

    def stats(self) -> st_plan_cache_stats:
        out = st_plan_cache_stats()
        _check(lib().st_plan_cache_get_stats(self.handle, ctypes.byref(out)), "st_plan_cache_get_stats")
        return out

    def destroy(self):
        if getattr(self, "handle", None) and _lib is not None:
            try:
                _lib.st_plan_cache_destroy(self.handle)
            except Exception:      # interpreter shutdown
                pass
            self.handle = None

    def __del__(self):
        self.destroy()


def make_chain_op(kind: int, sequence: int, stage: int, desc: st_conv_desc) -> st_chain_op:
    op = st_chain_op()
    op.kind, op.sequence, op.stage, op.reserved = kind, sequence, stage, 0
    op.conv = desc
    return op


class Chain:
    """Owns an st_chain*; keeps the tensors it borrows alive."""

    def __init__(self, ops: Sequence[st_chain_op], opts: Optional[st_plan_opts] = None, keep=None):
        n = len(ops)
        arr = (st_chain_op * max(n, 1))(*ops)
        out = ctypes.c_void_p()
        _check(lib().st_chain_plan(arr, n, ctypes.byref(opts) if opts is not None else None, ctypes.byref(out)), "st_chain_plan")
        self.handle, self._keep = out.value, keep

    def run(self, stream=None) -> None:
        _check(lib().st_chain_run(self.handle, _stream(stream)), "st_chain_run")

    def run_profiled(self, stream=None) -> np.ndarray:
        n = int(self.info().n_items)
        out = np.zeros((max(n, 1), 8), dtype=np.uint64)
        _check(lib().st_chain_run_profiled(self.handle, _stream(stream), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), out.size),
               "st_chain_run_profiled")
        return out[:n]

    def aborted(self) -> bool:
        flag = ctypes.c_int32()
        _check(lib().st_chain_aborted(self.handle, ctypes.byref(flag)), "st_chain_aborted")
        return bool(flag.value)

    def set_wait_limit_us(self, us: int) -> None:
        _check(lib().st_chain_set_wait_limit_us(self.handle, us), "st_chain_set_wait_limit_us")

    def info(self) -> st_chain_info:
        out = st_chain_info()
        _check(lib().st_chain_get_info(self.handle, ctypes.byref(out)), "st_chain_get_info")
        return out

    def op_info(self, op: int) -> st_chain_op_info:
        out = st_chain_op_info()
        _check(lib().st_chain_get_op_info(self.handle, op, ctypes.byref(out)), "st_chain_get_op_info")
        return out

    def worklist(self) -> np.ndarray:
        p = ctypes.POINTER(st_work_item)()
        n = ctypes.c_int64()
        _check(lib().st_chain_worklist(self.handle, ctypes.byref(p), ctypes.byref(n)), "st_chain_worklist")
        if n.value == 0:
            return np.zeros(0, dtype=WORK_ITEM_DTYPE)
        return np.frombuffer(ctypes.string_at(p, n.value * ctypes.sizeof(st_work_item)), dtype=WORK_ITEM_DTYPE).copy()

    def set_workgroups(self, n: int) -> None:
        _check(lib().st_chain_set_workgroups(self.handle, int(n)), "st_chain_set_workgroups")

    def columns(self) -> np.ndarray:
        """Column boundaries (8 * 2 * info().columns + 1 entries; empty with one queue), see st_chain_columns."""
        p = ctypes.POINTER(ctypes.c_uint32)()
        n = ctypes.c_int64()
        _check(lib().st_chain_columns(self.handle, ctypes.byref(p), ctypes.byref(n)), "st_chain_columns")
        if n.value == 0:
            return np.zeros(0, dtype=np.uint32)
        return np.frombuffer(ctypes.string_at(p, n.value * 4), dtype=np.uint32).copy()

    def destroy(self):
        if getattr(self, "handle", None) and _lib is not None:
            try:
                _lib.st_chain_destroy(self.handle)
            except Exception:      # interpreter shutdown
                pass
            self.handle = None

    def __del__(self):
        self.destroy()


def st_conv_plan_info(plan: Plan) -> st_plan_info:
    out = st_plan_info()
    _check(lib().st_conv_plan_info(plan.handle, ctypes.byref(out)), "st_conv_plan_info")
    return out


def st_conv_plan_tenant_info(plan: Plan, tenant: int) -> st_tenant_info:
    out = st_tenant_info()
    _check(lib().st_conv_plan_tenant_info(plan.handle, tenant, ctypes.byref(out)), "st_conv_plan_tenant_info")
    return out


def st_conv_plan_worklist(plan: Plan, which: int = 0) -> np.ndarray:
    """Copy of a work list as a structured array (fields as in st_work_item)."""
    p = ctypes.POINTER(st_work_item)()
    n = ctypes.c_int64()
    _check(lib().st_conv_plan_worklist(plan.handle, which, ctypes.byref(p), ctypes.byref(n)), "st_conv_plan_worklist")
    if n.value == 0:
        return np.zeros(0, dtype=WORK_ITEM_DTYPE)
    buf = ctypes.string_at(p, n.value * ctypes.sizeof(st_work_item))
    return np.frombuffer(buf, dtype=WORK_ITEM_DTYPE).copy()


def st_tile_shape(index: int):
    mt, nt, kb = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().st_tile_shape(index, ctypes.byref(mt), ctypes.byref(nt), ctypes.byref(kb)), "st_tile_shape")
    return mt.value, nt.value, kb.value


def st_tile_count() -> int:
    return lib().st_tile_count()


def st_maxpool_nhwc(x, y, N, H, W, C, win, stride, pad, dtype, stream=None) -> None:
    _check(lib().st_maxpool_nhwc(_ptr(x), _ptr(y), N, H, W, C, win, stride, pad, DTYPE_CODE.get(dtype, dtype),
                                 _stream(stream)), "st_maxpool_nhwc")


def st_launch_copy(src, dst, nbytes: int, stream=None) -> None:
    _check(lib().st_launch_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "st_launch_copy")


def st_launch_empty(stream=None) -> None:
    _check(lib().st_launch_empty(_stream(stream)), "st_launch_empty")
