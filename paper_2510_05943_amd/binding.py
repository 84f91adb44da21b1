"""ctypes binding of libearl_dispatch.so: same calls as include/earl_dispatch.h.

Only argument marshalling happens here (tensors -> device pointers, Python lists -> C arrays,
host result buffers -> numpy arrays).  Every step of the path runs in the library's kernels.
Device memory and streams come from the caller (PyTorch tensors / torch.cuda streams, or
anything with a `data_ptr()`); there is no CPU fallback: if the library has not been built,
the first call raises.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libearl_dispatch.so")

EARL_OK, EARL_INVALID_ARG, EARL_SEQ_EXCEEDS_BUDGET, EARL_CAPACITY, EARL_HIP_ERROR = range(5)
EARL_MAX_FIELDS = 32

EXPORTED = ("earl_plan_workspace_bytes", "earl_plan_build", "earl_plan_get_summary",
            "earl_plan_export", "earl_plan_export_segments", "earl_dispatch_workspace_bytes",
            "earl_dispatch", "earl_dispatch_async_workspace_bytes", "earl_dispatch_async",
            "earl_dispatch_async_status", "earl_dispatch_noalloc",
            "earl_dispatch_inverse", "earl_plan_set_dispatch_events", "earl_plan_destroy", "earl_status_string",
            "earl_last_error_message")


class EarlError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"earl status {status}: {message}")
        self.status = status


class _SrcLayout(C.Structure):
    _fields_ = [("n_groups", C.c_int32), ("replication", C.c_int32),
                ("seq_group", C.c_void_p), ("seq_row", C.c_void_p)]


class _DstLayout(C.Structure):
    _fields_ = [("dp", C.c_int32), ("sp", C.c_int32), ("zigzag", C.c_int32),
                ("pad_multiple", C.c_int32), ("balance_policy", C.c_int32),
                ("equal_mb", C.c_int32), ("mb_token_budget", C.c_int64)]


class _Field(C.Structure):
    _fields_ = [("scalar_bytes", C.c_int32), ("width", C.c_int32), ("pad_scalar", C.c_uint64),
                ("src_shard_ptrs", C.POINTER(C.c_void_p)), ("dst_shard_ptrs", C.POINTER(C.c_void_p)),
                ("dst_capacity_rows", C.POINTER(C.c_int64)),
                ("src_capacity_rows", C.POINTER(C.c_int64)),
                ("per_sequence", C.c_int32), ("nonzero_counts", C.c_void_p),
                ("nonzero_counts_capacity", C.c_int64)]


class _Summary(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_src_shards", C.c_int32), ("n_dst_shards", C.c_int32),
                ("chunks_per_seq", C.c_int32), ("n_segments", C.c_int32), ("n_mb_max", C.c_int32),
                ("cu_seqlens_len", C.c_int32), ("mb_table_len", C.c_int32),
                ("total_real_rows", C.c_int64), ("total_dst_rows", C.c_int64),
                ("rank_load_min", C.c_int64), ("rank_load_max", C.c_int64),
                ("shard_rows", C.POINTER(C.c_int64)), ("src_rows_needed", C.POINTER(C.c_int64)),
                ("src_seqs_needed", C.POINTER(C.c_int64)),
                ("n_seq", C.POINTER(C.c_int32)), ("n_mb", C.POINTER(C.c_int32)),
                ("rank_load", C.POINTER(C.c_int64)), ("a2a_counts", C.POINTER(C.c_int64))]


_lib = None


def load_library() -> C.CDLL:
    """Loads the built library (no GPU needed for loading).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2510_05943_amd.build` "
            "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.earl_plan_workspace_bytes.argtypes = [i32, C.POINTER(_SrcLayout), C.POINTER(_DstLayout),
                                              C.POINTER(C.c_size_t)]
    lib.earl_plan_build.argtypes = [vp, i32, C.POINTER(_SrcLayout), C.POINTER(_DstLayout), vp,
                                    C.c_size_t, vp, C.POINTER(vp)]
    lib.earl_plan_get_summary.argtypes = [vp, C.POINTER(_Summary)]
    lib.earl_plan_export.argtypes = [vp] + [vp] * 10
    lib.earl_plan_export_segments.argtypes = [vp] + [vp] * 8
    lib.earl_dispatch_workspace_bytes.argtypes = [vp, C.POINTER(_Field), i32, i32, i32,
                                                  C.POINTER(C.c_size_t)]
    lib.earl_dispatch.argtypes = [vp, C.POINTER(_Field), i32, C.POINTER(vp), vp, vp, C.c_size_t, vp]
    lib.earl_dispatch_async_workspace_bytes.argtypes = [vp, C.POINTER(_Field), i32, vp, i64,
                                                        C.POINTER(C.c_size_t)]
    lib.earl_dispatch_async.argtypes = [vp, C.POINTER(_Field), i32, C.POINTER(vp), vp, vp, i64, vp,
                                        C.c_size_t, vp]
    lib.earl_dispatch_async_status.argtypes = [vp, C.POINTER(i32)]
    lib.earl_dispatch_noalloc.argtypes = [vp, C.POINTER(_Field), i32, C.POINTER(vp), vp, vp]
    lib.earl_dispatch_inverse.argtypes = [vp, C.POINTER(_Field), i32, vp, C.c_size_t, vp]
    lib.earl_plan_set_dispatch_events.argtypes = [vp, vp, vp]
    lib.earl_plan_destroy.argtypes = [vp]
    lib.earl_status_string.argtypes = [i32]
    lib.earl_status_string.restype = C.c_char_p
    lib.earl_last_error_message.argtypes = []
    lib.earl_last_error_message.restype = C.c_char_p
    for name in EXPORTED:
        if name not in ("earl_status_string", "earl_last_error_message"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != EARL_OK:
        lib = load_library()
        msg = lib.earl_last_error_message().decode() or lib.earl_status_string(status).decode()
        raise EarlError(status, msg)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


@dataclasses.dataclass
class SrcLayout:
    n_groups: int
    replication: int = 1
    seq_group: object = None   # device int32[N] tensor or None
    seq_row: object = None     # device int64[N] tensor or None

    def c(self) -> _SrcLayout:
        return _SrcLayout(self.n_groups, self.replication, _ptr(self.seq_group), _ptr(self.seq_row))


@dataclasses.dataclass
class DstLayout:
    dp: int
    sp: int = 1
    zigzag: int = 0
    pad_multiple: int = 1
    mb_token_budget: int = 1 << 40
    balance_policy: int = 0
    equal_mb: int = 0

    def c(self) -> _DstLayout:
        return _DstLayout(self.dp, self.sp, self.zigzag, self.pad_multiple, self.balance_policy,
                          self.equal_mb, self.mb_token_budget)


@dataclasses.dataclass
class Field:
    """One field: per-shard device buffers in both layouts.  Buffers are tensors (or objects
    with data_ptr()/numel()/element_size()); None marks a shard without a buffer.  The C
    descriptor is built at the first call and kept: do not change a Field after using it."""
    scalar_bytes: int
    width: int
    pad_scalar: int
    src_shards: Sequence
    dst_shards: Sequence
    check_src_capacity: bool = True
    per_sequence: bool = False     # source holds one row per sequence, broadcast to its tokens
    nonzero_counts: object = None  # int64 tensor [D*C * n_mb_max]: non-zero scalars per micro-batch

    def _rows(self, t) -> int:
        row_bytes = self.scalar_bytes * self.width
        if t is None or row_bytes <= 0:
            return 0
        return (int(t.numel()) * int(t.element_size())) // row_bytes


@dataclasses.dataclass
class Plan:
    handle: int
    workspace: object
    src: SrcLayout
    dst: DstLayout
    n_seqs: int
    keepalive: tuple = ()


def plan_workspace_bytes(n_seqs: int, src: SrcLayout, dst: DstLayout) -> int:
    out = C.c_size_t(0)
    s, d = src.c(), dst.c()
    _check(load_library().earl_plan_workspace_bytes(n_seqs, C.byref(s), C.byref(d), C.byref(out)))
    return int(out.value)


def plan_build(lengths_dev, n_seqs: int, src: SrcLayout, dst: DstLayout, workspace,
               workspace_bytes: Optional[int] = None, stream=None) -> Plan:
    """earl_plan_build.  `workspace` is a device tensor (or pointer) owned by the caller."""
    if workspace_bytes is None:
        workspace_bytes = int(workspace.numel()) * int(workspace.element_size())
    s, d = src.c(), dst.c()
    handle = C.c_void_p(None)
    _check(load_library().earl_plan_build(_ptr(lengths_dev), n_seqs, C.byref(s), C.byref(d),
                                          _ptr(workspace), workspace_bytes,
                                          _stream_handle(stream), C.byref(handle)))
    return Plan(handle.value, workspace, src, dst, n_seqs, keepalive=(lengths_dev,))


def plan_get_summary(plan: Plan) -> Dict:
    s = _Summary()
    _check(load_library().earl_plan_get_summary(plan.handle, C.byref(s)))
    n_dst, n_src, dp = s.n_dst_shards, s.n_src_shards, plan.dst.dp
    out = {k: int(getattr(s, k)) for k in
           ("n_seqs", "n_src_shards", "n_dst_shards", "chunks_per_seq", "n_segments", "n_mb_max",
            "cu_seqlens_len", "mb_table_len", "total_real_rows", "total_dst_rows",
            "rank_load_min", "rank_load_max")}
    def arr(ptr, n, dtype):
        # a host copy of n entries (string_at + frombuffer is 2-3x cheaper than ctypeslib.as_array)
        return np.frombuffer(C.string_at(ptr, n * np.dtype(dtype).itemsize), dtype=dtype).copy()

    out["shard_rows"] = arr(s.shard_rows, n_dst, np.int64)
    out["src_rows_needed"] = arr(s.src_rows_needed, n_src, np.int64)
    out["src_seqs_needed"] = arr(s.src_seqs_needed, n_src, np.int64)
    out["n_seq"] = arr(s.n_seq, dp, np.int32)
    out["n_mb"] = arr(s.n_mb, dp, np.int32)
    out["rank_load"] = arr(s.rank_load, dp, np.int64)
    out["a2a_counts"] = arr(s.a2a_counts, n_src * n_dst, np.int64).reshape(n_src, n_dst)
    return out


def plan_wait(plan: Plan) -> int:
    """earl_plan_get_summary without host copies of its arrays: returns (with n_mb_max) once the
    plan's totals are on the host, which is all a loop with pre-allocated buffers needs
    between earl_plan_build and earl_dispatch."""
    s = _Summary()
    _check(load_library().earl_plan_get_summary(plan.handle, C.byref(s)))
    return int(s.n_mb_max)


def plan_export(plan: Plan) -> Dict[str, np.ndarray]:
    sm = plan_get_summary(plan)
    n = plan.n_seqs
    bufs = dict(rank=np.empty(n, np.int32), slot=np.empty(n, np.int32), mb=np.empty(n, np.int32),
                dst_row=np.empty(n, np.int64), seq_shard=np.empty(n, np.int32),
                seq_row=np.empty(n, np.int64), seq_ids=np.empty(n, np.int32),
                mb_seq_start=np.empty(sm["mb_table_len"], np.int32),
                mb_row_start=np.empty(sm["mb_table_len"], np.int64),
                cu_seqlens=np.empty(sm["cu_seqlens_len"], np.int32))
    order = ("rank", "slot", "mb", "dst_row", "seq_shard", "seq_row", "seq_ids", "mb_seq_start",
             "mb_row_start", "cu_seqlens")
    _check(load_library().earl_plan_export(plan.handle, *[bufs[k].ctypes.data for k in order]))
    return bufs


def plan_export_segments(plan: Plan) -> Dict[str, np.ndarray]:
    sm = plan_get_summary(plan)
    e = sm["n_segments"]
    bufs = dict(src_shard=np.empty(e, np.int32), src_row=np.empty(e, np.int64),
                dst_shard=np.empty(e, np.int32), dst_row=np.empty(e, np.int64),
                n_real=np.empty(e, np.int32), n_rows=np.empty(e, np.int32),
                pos0=np.empty(e, np.int32),
                shard_seg_start=np.empty(sm["n_dst_shards"] + 1, np.int32))
    order = ("src_shard", "src_row", "dst_shard", "dst_row", "n_real", "n_rows", "pos0",
             "shard_seg_start")
    _check(load_library().earl_plan_export_segments(plan.handle,
                                                    *[bufs[k].ctypes.data for k in order]))
    return bufs


def _marshal_field(f: Field):
    """C descriptor of one field; built once per Field object and kept with it."""
    cached = getattr(f, "_c", None)
    if cached is not None:
        return cached
    src = (C.c_void_p * len(f.src_shards))(*[_ptr(t) for t in f.src_shards])
    dst = (C.c_void_p * len(f.dst_shards))(*[_ptr(t) for t in f.dst_shards])
    cap = (C.c_int64 * len(f.dst_shards))(*[f._rows(t) for t in f.dst_shards])
    scap = (C.c_int64 * len(f.src_shards))(*[f._rows(t) for t in f.src_shards])
    desc = _Field(f.scalar_bytes, f.width, f.pad_scalar & 0xFFFFFFFFFFFFFFFF,
                  C.cast(src, C.POINTER(C.c_void_p)), C.cast(dst, C.POINTER(C.c_void_p)),
                  C.cast(cap, C.POINTER(C.c_int64)),
                  C.cast(scap, C.POINTER(C.c_int64)) if f.check_src_capacity else None,
                  1 if f.per_sequence else 0, _ptr(f.nonzero_counts),
                  0 if f.nonzero_counts is None else int(f.nonzero_counts.numel()))
    f._c = (desc, (src, dst, cap, scap))
    return f._c


def _marshal_fields(fields: Sequence[Field]):
    n = len(fields)
    arr = (_Field * max(n, 1))()
    keep = []
    for k, f in enumerate(fields):
        desc, owned = _marshal_field(f)
        arr[k] = desc
        keep.append(owned)
    return arr, n, keep


def _nbytes(t) -> int:
    return 0 if t is None else int(t.numel()) * int(t.element_size())


def dispatch_workspace_bytes(plan: Plan, fields: Sequence[Field], with_position_ids: bool = True,
                             with_cu_seqlens: bool = True) -> int:
    """earl_dispatch_workspace_bytes: scratch one dispatch call with these fields needs."""
    arr, n, keep = _marshal_fields(fields)
    out = C.c_size_t(0)
    _check(load_library().earl_dispatch_workspace_bytes(plan.handle, arr, n, int(with_position_ids),
                                                        int(with_cu_seqlens), C.byref(out)))
    return int(out.value)


def dispatch(plan: Plan, fields: Sequence[Field], position_ids: Optional[Sequence] = None,
             cu_seqlens=None, workspace=None, stream=None) -> None:
    """earl_dispatch: materialise all destination shards (asynchronous on the stream).
    `workspace` is a device buffer of at least dispatch_workspace_bytes() bytes."""
    arr, n, keep = _marshal_fields(fields)
    pos = None
    if position_ids is not None:
        pos = (C.c_void_p * len(position_ids))(*[_ptr(t) for t in position_ids])
    _check(load_library().earl_dispatch(plan.handle, arr, n,
                                        C.cast(pos, C.POINTER(C.c_void_p)) if pos is not None else None,
                                        _ptr(cu_seqlens), _ptr(workspace), _nbytes(workspace),
                                        _stream_handle(stream)))


def dispatch_noalloc(plan: Plan, fields: Sequence[Field], position_ids: Optional[Sequence] = None,
                     cu_seqlens=None, stream=None) -> None:
    """earl_dispatch_noalloc: earl_dispatch on the library's own fixed scratch array; the plan's
    summary must have been fetched."""
    arr, n, keep = _marshal_fields(fields)
    pos = None
    if position_ids is not None:
        pos = (C.c_void_p * len(position_ids))(*[_ptr(t) for t in position_ids])
    _check(load_library().earl_dispatch_noalloc(
        plan.handle, arr, n, C.cast(pos, C.POINTER(C.c_void_p)) if pos is not None else None,
        _ptr(cu_seqlens), _stream_handle(stream)))


def _capacity_array(tensors: Optional[Sequence]):
    if tensors is None:
        return None
    return (C.c_int64 * len(tensors))(*[0 if t is None else int(t.numel()) for t in tensors])


def dispatch_async_workspace_bytes(plan: Plan, fields: Sequence[Field],
                                   position_ids: Optional[Sequence] = None, cu_seqlens=None) -> int:
    """earl_dispatch_async_workspace_bytes; capacities are taken from the buffers' sizes."""
    arr, n, keep = _marshal_fields(fields)
    out = C.c_size_t(0)
    _check(load_library().earl_dispatch_async_workspace_bytes(
        plan.handle, arr, n, _capacity_array(position_ids),
        0 if cu_seqlens is None else int(cu_seqlens.numel()), C.byref(out)))
    return int(out.value)


def dispatch_async(plan: Plan, fields: Sequence[Field], position_ids: Optional[Sequence] = None,
                   cu_seqlens=None, workspace=None, stream=None) -> None:
    """earl_dispatch_async: enqueued behind the plan without waiting for it.  Position-id buffers
    are int32 tensors (capacity = their element count), as is cu_seqlens."""
    arr, n, keep = _marshal_fields(fields)
    pos = None
    if position_ids is not None:
        pos = (C.c_void_p * len(position_ids))(*[_ptr(t) for t in position_ids])
    _check(load_library().earl_dispatch_async(
        plan.handle, arr, n, pos, _capacity_array(position_ids), _ptr(cu_seqlens),
        0 if cu_seqlens is None else int(cu_seqlens.numel()), _ptr(workspace), _nbytes(workspace),
        _stream_handle(stream)))


def dispatch_async_status(plan: Plan) -> int:
    """earl_dispatch_async_status: waits for the stream; EARL_OK if the last call was carried out."""
    st = C.c_int32(-1)
    _check(load_library().earl_dispatch_async_status(plan.handle, C.byref(st)))
    return st.value


def dispatch_inverse(plan: Plan, fields: Sequence[Field], workspace=None, stream=None) -> None:
    """earl_dispatch_inverse: copy every real row back to the rollout layout."""
    arr, n, keep = _marshal_fields(fields)
    _check(load_library().earl_dispatch_inverse(plan.handle, arr, n, _ptr(workspace),
                                                _nbytes(workspace), _stream_handle(stream)))


def plan_set_dispatch_events(plan: Plan, event_before: Optional[int], event_after: Optional[int]) -> None:
    """earl_plan_set_dispatch_events: raw hipEvent_t handles (ints) or None, None."""
    _check(load_library().earl_plan_set_dispatch_events(plan.handle, event_before, event_after))


def plan_destroy(plan: Plan) -> None:
    if plan.handle:
        _check(load_library().earl_plan_destroy(plan.handle))
        plan.handle = None
