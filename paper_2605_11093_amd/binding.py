"""ctypes binding of include/dmi.h: same names, argument marshalling only.

Every step of the capture-and-stage path runs inside libdmi.so.  There is no
fallback: if the library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdmi.so")
_lib = None

OK, SAMPLED_OUT, POINT_DISABLED = 0, 1, 2
ERR_INVALID_ARG, ERR_NOMEM, ERR_TOO_LARGE, ERR_HIP, ERR_AGAIN, ERR_CLOSED = -1, -2, -3, -4, -5, -6
DT_NONE, DT_BF16, DT_FP16, DT_FP32, DT_FP8 = 0, 1, 2, 3, 4
SUM_L2, SUM_MEAN, SUM_ABSMAX = 1, 2, 4
POLICY_BLOCK, POLICY_DROP_NEWEST = 0, 1
DRAIN_COPY_ENGINE, DRAIN_KERNEL, BG_THREAD = 1, 2, 4
DRAIN_NONBLOCK, DRAIN_FLUSH = 1, 2


class DmiError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dmi error {code}: {msg}")
        self.code = code


class RingConfig(C.Structure):
    _fields_ = [("device_ring_bytes", C.c_uint64), ("host_ring_bytes", C.c_uint64),
                ("device_id", C.c_int32), ("flags", C.c_uint32),
                ("max_reqs_per_observe", C.c_uint32), ("rank_tag", C.c_uint32),
                ("bg_min_bytes", C.c_uint64), ("bg_timeout_us", C.c_uint32),
                ("block_timeout_ms", C.c_uint32), ("bg_min_records", C.c_uint32),
                ("bg_occupancy_pct", C.c_uint32)]


class Tensor(C.Structure):
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_uint32), ("shape", C.c_int64 * 2),
                ("stride", C.c_int64 * 2)]


class ReqSel(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("req_id", "row_base", "tok_start", "tok_count", "tok_step")]


class Selection(C.Structure):
    _fields_ = [("n_reqs", C.c_uint32), ("reqs", C.c_void_p), ("keep_mask_dev", C.c_void_p),
                ("row_index_dev", C.c_void_p)]


class Transform(C.Structure):
    _fields_ = [("out_dtype", C.c_uint32), ("summary_mask", C.c_uint32)]


class PagedKV(C.Structure):
    _fields_ = [("base", C.c_void_p), ("dtype", C.c_uint32), ("block_stride", C.c_int64),
                ("slot_stride", C.c_int64), ("head_stride", C.c_int64),
                ("block_size", C.c_uint32), ("n_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("n_blocks", C.c_uint32), ("n_seqs", C.c_uint32),
                ("block_table_dev", C.c_void_p), ("block_table_stride", C.c_int64),
                ("n_heads_sel", C.c_uint32), ("heads_sel", C.c_uint32 * 8)]


class RecordViewC(C.Structure):
    _fields_ = [("p0", C.c_void_p), ("n0", C.c_uint64), ("p1", C.c_void_p), ("n1", C.c_uint64),
                ("seq", C.c_uint64)]


class ReqInfo(C.Structure):
    _fields_ = [("req_id", C.c_uint32), ("rows", C.c_uint32), ("admit_order", C.c_uint64),
                ("matches", C.c_uint32), ("reserved", C.c_uint32)]


class SliceC(C.Structure):
    _fields_ = [("seq", C.c_uint64), ("step_id", C.c_uint64), ("point_id", C.c_uint32), ("rank_tag", C.c_uint32),
                ("req_index", C.c_uint32), ("req_id", C.c_uint32), ("tok_start", C.c_uint32),
                ("tok_step", C.c_uint32), ("n_rows", C.c_uint32), ("row_elems", C.c_uint32),
                ("src_dtype", C.c_uint32), ("out_dtype", C.c_uint32), ("summary_mask", C.c_uint32),
                ("flags", C.c_uint32), ("rows", C.c_void_p), ("l2", C.c_void_p), ("mean", C.c_void_p),
                ("absmax", C.c_void_p), ("owner", C.c_void_p)]


class Policy(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("sample_k", C.c_uint32), ("sample_phase", C.c_uint32)]


_STAT_FIELDS = ("observed_calls", "launched_records", "captured_records", "captured_rows",
                "captured_bytes", "dropped_records", "dropped_rows", "dropped_bytes",
                "sampled_out_calls", "sampled_out_rows", "disabled_calls", "drained_bytes",
                "released_bytes", "drain_batches", "block_wait_ns", "dev_ring_high_water",
                "host_ring_high_water", "bad_rows")


class StatsC(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in _STAT_FIELDS]


@dataclass
class Stats:
    observed_calls: int = 0
    launched_records: int = 0
    captured_records: int = 0
    captured_rows: int = 0
    captured_bytes: int = 0
    dropped_records: int = 0
    dropped_rows: int = 0
    dropped_bytes: int = 0
    sampled_out_calls: int = 0
    sampled_out_rows: int = 0
    disabled_calls: int = 0
    drained_bytes: int = 0
    released_bytes: int = 0
    drain_batches: int = 0
    block_wait_ns: int = 0
    dev_ring_high_water: int = 0
    host_ring_high_water: int = 0
    bad_rows: int = 0


@dataclass
class RecordView:
    seq: int
    p0: int
    n0: int
    p1: int
    n1: int

    @property
    def nbytes(self) -> int:
        return self.n0 + self.n1

    def bytes(self) -> np.ndarray:
        """Copy of the record's bytes (valid only until the record is released)."""
        out = np.empty(self.n0 + self.n1, dtype=np.uint8)
        C.memmove(out.ctypes.data, self.p0, self.n0)
        if self.n1:
            C.memmove(out.ctypes.data + self.n0, self.p1, self.n1)
        return out


def library_path() -> str:
    return _SO


def lib():
    """Load libdmi.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_SO):
        raise ImportError(f"{_SO} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(_SO)
    P = C.POINTER
    L.dmi_last_error.restype = C.c_char_p
    L.dmi_version.restype = C.c_char_p
    L.dmi_record_bytes.restype = C.c_uint64
    L.dmi_record_bytes.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
    L.dmi_ring_create.argtypes = [P(RingConfig), P(C.c_void_p)]
    L.dmi_ring_destroy.argtypes = [C.c_void_p]
    L.dmi_observe.argtypes = [C.c_void_p, C.c_uint32, P(Tensor), P(Selection), P(Transform),
                              C.c_uint64, C.c_void_p]
    L.dmi_observe_paged.argtypes = [C.c_void_p, C.c_uint32, P(PagedKV), P(Selection), P(Transform),
                                    C.c_uint64, C.c_void_p]
    L.dmi_observe_batch.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint32), P(C.c_void_p), P(Tensor), P(Selection),
                                    P(Transform), C.c_uint64, C.c_void_p, P(C.c_uint32)]
    L.dmi_observe_paged_batch.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint32), P(C.c_void_p), P(PagedKV),
                                          P(Selection), P(Transform), C.c_uint64, C.c_void_p, P(C.c_uint32)]
    L.dmi_step_observe_batch.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint32), P(C.c_void_p), P(Tensor),
                                         P(Selection), P(Transform), C.c_void_p, P(C.c_uint32)]
    L.dmi_step_observe_paged_batch.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint32), P(C.c_void_p), P(PagedKV),
                                               P(Selection), P(Transform), C.c_void_p, P(C.c_uint32)]
    for name in ("dmi_observe_batch", "dmi_observe_paged_batch", "dmi_step_observe_batch",
                 "dmi_step_observe_paged_batch"):
        getattr(L, name).restype = C.c_int32
    L.dmi_observe_into.argtypes = [C.c_uint32, P(Tensor), P(Selection), P(Transform), C.c_uint64, C.c_uint64,
                                   C.c_uint32, C.c_void_p, C.c_uint64, P(C.c_uint64), C.c_void_p]
    L.dmi_observe_into.restype = C.c_int32
    L.dmi_drain.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint64)]
    L.dmi_poll_host.argtypes = [C.c_void_p, P(RecordViewC), C.c_uint32, P(C.c_uint32)]
    L.dmi_release_host.argtypes = [C.c_void_p, C.c_uint64]
    L.dmi_set_policy.argtypes = [C.c_void_p, P(Policy)]
    L.dmi_point_enable.argtypes = [C.c_void_p, C.c_uint32, C.c_int]
    L.dmi_get_stats.argtypes = [C.c_void_p, P(StatsC)]
    L.dmi_get_point_drops.argtypes = [C.c_void_p, C.c_uint32, P(C.c_uint64)]
    L.dmi_debug_fill_rings.argtypes = [C.c_void_p, C.c_uint8]
    L.dmi_debug_exporter_allocs.argtypes = [C.c_void_p, P(C.c_uint64), P(C.c_uint64)]
    L.dmi_debug_exporter_allocs.restype = C.c_int32
    L.dmi_debug_time_next_launch.argtypes = [C.c_void_p, C.c_void_p]
    L.dmi_debug_time_next_launch.restype = C.c_int32
    L.dmi_exporter_start.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32]
    L.dmi_exporter_next.argtypes = [C.c_void_p, P(SliceC), C.c_uint32]
    L.dmi_exporter_release.argtypes = [C.c_void_p, P(SliceC)]
    L.dmi_exporter_next_many.argtypes = [C.c_void_p, P(SliceC), C.c_uint32, P(C.c_uint32), C.c_uint32]
    L.dmi_exporter_release_many.argtypes = [C.c_void_p, P(SliceC), C.c_uint32]
    L.dmi_exporter_stop.argtypes = [C.c_void_p]
    L.dmi_policy_select.argtypes = [C.c_uint32, P(ReqInfo), C.c_uint32, C.c_uint64, C.c_uint64, C.c_void_p,
                                    P(C.c_uint32)]
    L.dmi_ring_free_bytes.argtypes = [C.c_void_p, P(C.c_uint64)]
    L.dmi_set_keep_mask.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, P(C.c_void_p)]
    L.dmi_step_create.argtypes = [C.c_void_p, C.c_uint32, P(C.c_void_p)]
    L.dmi_step_destroy.argtypes = [C.c_void_p]
    L.dmi_step_capture_begin.argtypes = [C.c_void_p]
    L.dmi_step_observe.argtypes = [C.c_void_p, C.c_uint32, P(Tensor), P(Selection), P(Transform), C.c_void_p,
                                   P(C.c_uint32)]
    L.dmi_step_observe_paged.argtypes = [C.c_void_p, C.c_uint32, P(PagedKV), P(Selection), P(Transform),
                                         C.c_void_p, P(C.c_uint32)]
    L.dmi_step_seal.argtypes = [C.c_void_p]
    L.dmi_step_update.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32]
    L.dmi_step_begin.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
    L.dmi_step_end.argtypes = [C.c_void_p, C.c_void_p]
    for name in ("dmi_step_create", "dmi_step_destroy", "dmi_step_capture_begin", "dmi_step_observe",
                 "dmi_step_observe_paged", "dmi_step_seal", "dmi_step_update", "dmi_step_begin", "dmi_step_end"):
        getattr(L, name).restype = C.c_int32
    for name in ("dmi_ring_create", "dmi_ring_destroy", "dmi_observe", "dmi_observe_paged", "dmi_drain",
                 "dmi_poll_host", "dmi_release_host", "dmi_set_policy", "dmi_point_enable",
                 "dmi_get_stats", "dmi_get_point_drops", "dmi_debug_fill_rings", "dmi_policy_select",
                 "dmi_ring_free_bytes", "dmi_set_keep_mask", "dmi_exporter_start", "dmi_exporter_next",
                 "dmi_exporter_release", "dmi_exporter_stop", "dmi_exporter_next_many",
                 "dmi_exporter_release_many"):
        getattr(L, name).restype = C.c_int32
    _lib = L
    return L


def version() -> str:
    return lib().dmi_version().decode()


def record_bytes(n_reqs: int, n_rows: int, row_elems: int, out_dtype: int, summary_mask: int) -> int:
    return int(lib().dmi_record_bytes(n_reqs, n_rows, row_elems, out_dtype, summary_mask))


SELECT_DROP_RECENT, SELECT_KEEP_BY_PATTERN = 0, 1


def policy_select(strategy: int, reqs, bytes_per_row: int, budget_bytes: int) -> np.ndarray:
    """reqs: iterable of (req_id, rows, admit_order, matches).  Returns the keep vector (uint8)."""
    rows = list(reqs)
    arr = (ReqInfo * max(1, len(rows)))(*[ReqInfo(int(a), int(b), int(c), int(d), 0) for a, b, c, d in rows])
    keep = np.zeros(len(rows), dtype=np.uint8)
    n = C.c_uint32()
    _check(lib().dmi_policy_select(strategy, arr, len(rows), bytes_per_row, budget_bytes,
                                   keep.ctypes.data if len(rows) else None, C.byref(n)))
    assert int(n.value) == int(keep.sum())
    return keep


def _check(code: int, allow: Sequence[int] = ()) -> int:
    if code < 0 and code not in allow:
        raise DmiError(code, lib().dmi_last_error().decode())
    return code


_TORCH_DT = None


def _torch_dtype_code(t) -> int:
    global _TORCH_DT
    if _TORCH_DT is None:
        import torch
        _TORCH_DT = {torch.bfloat16: DT_BF16, torch.float16: DT_FP16, torch.float32: DT_FP32}
    return _TORCH_DT[t.dtype]


def time_next_launch(start_event: int, stop_event: int) -> None:
    """The calling thread's next capture launch records its own start and end into the two hipEvent_t handles."""
    _check(lib().dmi_debug_time_next_launch(start_event or None, stop_event or None))


def _reqs_buffer(reqs):
    a = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
    return a


def observe_into(point_id: int, tensor, reqs, out, *, seq: int, step_id: int, rank_tag: int = 0,
                 out_dtype: Optional[int] = None, summary_mask: int = 0, keep_mask=None, row_index=None,
                 stream: int = 0, allow: Sequence[int] = ()) -> int:
    """dmi_observe_into: one record into `out` (a uint8 device tensor), no ring, no allocation.
    Returns the record's size (an upper bound if a keep vector is given)."""
    dt = _torch_dtype_code(tensor)
    ra = _reqs_buffer(reqs)
    t = Tensor(tensor.data_ptr(), dt, (C.c_int64 * 2)(*tensor.shape), (C.c_int64 * 2)(*tensor.stride()))
    sel = Selection(ra.shape[0], ra.ctypes.data, None if keep_mask is None else keep_mask.data_ptr(),
                    None if row_index is None else row_index.data_ptr())
    xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
    n = C.c_uint64()
    _check(lib().dmi_observe_into(point_id, C.byref(t), C.byref(sel), C.byref(xf), seq, step_id, rank_tag,
                                  out.data_ptr(), out.numel() * out.element_size(), C.byref(n), stream or None),
           allow)
    return int(n.value)


class PreparedObserve:
    """The argument structs of one dmi_observe / dmi_observe_paged call, built once so
    that a per-step loop pays only the foreign call itself.  Calling it returns the
    raw status code."""

    def __init__(self, ring: "Ring", point_id: int, tensor, reqs, *, out_dtype: Optional[int] = None,
                 summary_mask: int = 0, keep_mask=None, row_index=None, paged=None):
        dt = _torch_dtype_code(tensor)
        self._keep = (tensor, keep_mask, row_index, paged)
        self._ra = _reqs_buffer(reqs)
        self._sel = Selection(self._ra.shape[0], self._ra.ctypes.data,
                              None if keep_mask is None else keep_mask.data_ptr(),
                              None if row_index is None else row_index.data_ptr())
        self._xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        self._h, self._point = ring._h, point_id
        if paged is None:
            self._src = Tensor(tensor.data_ptr(), dt, (C.c_int64 * 2)(*tensor.shape),
                               (C.c_int64 * 2)(*tensor.stride()))
            self._fn = lib().dmi_observe
        else:
            bt = paged.block_table
            self._src = PagedKV(tensor.data_ptr(), dt, tensor.stride(0), tensor.stride(1), tensor.stride(2),
                                paged.block_size, paged.n_heads, paged.head_dim, tensor.shape[0], bt.shape[0],
                                bt.data_ptr(), bt.stride(0), len(paged.heads_sel),
                                (C.c_uint32 * 8)(*paged.heads_sel))
            self._fn = lib().dmi_observe_paged
        self._a = (C.byref(self._src), C.byref(self._sel), C.byref(self._xf))

    def __call__(self, step_id: int, stream: int) -> int:
        return self._fn(self._h, self._point, self._a[0], self._a[1], self._a[2], step_id, stream)


def _paged_struct(cache, paged_or_table, *, block_size=None, n_heads=None, head_dim=None, heads_sel=None):
    """dmi_paged_kv_t for a cache tensor [blocks, slots, heads, dim]."""
    if block_size is None:
        p = paged_or_table
        bt, block_size, n_heads, head_dim, heads_sel = p.block_table, p.block_size, p.n_heads, p.head_dim, p.heads_sel
    else:
        bt = paged_or_table
    return PagedKV(cache.data_ptr(), _torch_dtype_code(cache), cache.stride(0), cache.stride(1), cache.stride(2),
                   block_size, n_heads, head_dim, cache.shape[0], bt.shape[0], bt.data_ptr(), bt.stride(0),
                   len(heads_sel), (C.c_uint32 * 8)(*heads_sel))


def _same_layout(tensors):
    t0 = tensors[0]
    for t in tensors[1:]:
        if t.dtype != t0.dtype or tuple(t.shape) != tuple(t0.shape) or tuple(t.stride()) != tuple(t0.stride()):
            raise ValueError("the tensors of a batch must share dtype, shape and strides")


class PreparedBatch:
    """The argument structs of one dmi_observe_batch / dmi_observe_paged_batch call, built once.
    Calling it returns (status, n_done)."""

    def __init__(self, ring: "Ring", point_ids, tensors, reqs, *, out_dtype: Optional[int] = None,
                 summary_mask: int = 0, keep_mask=None, row_index=None, paged=None):
        tensors = list(tensors)
        _same_layout(tensors)
        dt = _torch_dtype_code(tensors[0])
        self._keep = (tensors, keep_mask, row_index, paged)
        self._n = len(tensors)
        self._points = (C.c_uint32 * self._n)(*[int(p) for p in point_ids])
        self._data = (C.c_void_p * self._n)(*[t.data_ptr() for t in tensors])
        self._ra = _reqs_buffer(reqs)
        self._sel = Selection(self._ra.shape[0], self._ra.ctypes.data,
                              None if keep_mask is None else keep_mask.data_ptr(),
                              None if row_index is None else row_index.data_ptr())
        self._xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        self._h = ring._h
        t0 = tensors[0]
        if paged is None:
            self._like = Tensor(t0.data_ptr(), dt, (C.c_int64 * 2)(*t0.shape), (C.c_int64 * 2)(*t0.stride()))
            self._fn = lib().dmi_observe_batch
        else:
            self._like = _paged_struct(t0, paged)
            self._fn = lib().dmi_observe_paged_batch
        self._done = C.c_uint32()

    def __call__(self, step_id: int, stream: int):
        rc = self._fn(self._h, self._n, self._points, self._data, C.byref(self._like), C.byref(self._sel),
                      C.byref(self._xf), step_id, stream, C.byref(self._done))
        return rc, self._done.value


class Step:
    """A replayable step (dmi_step_*): capture launches that can sit in a captured graph."""

    def __init__(self, ring: "Ring", max_observes: int):
        h = C.c_void_p()
        _check(lib().dmi_step_create(ring._h, max_observes, C.byref(h)))
        self._h = h
        self._ring = ring

    def destroy(self):
        if self._h:
            _check(lib().dmi_step_destroy(self._h))
            self._h = None

    def capture_begin(self):
        _check(lib().dmi_step_capture_begin(self._h))

    def observe_tensor(self, point_id: int, tensor, reqs, *, stream: int, out_dtype: Optional[int] = None,
                       summary_mask: int = 0, keep_mask=None, row_index=None, allow: Sequence[int] = ()) -> int:
        """Returns the node index, or -1 if the point is disabled (nothing launched)."""
        dt = _torch_dtype_code(tensor)
        ra = _reqs_buffer(reqs)
        t = Tensor(tensor.data_ptr(), dt, (C.c_int64 * 2)(*tensor.shape), (C.c_int64 * 2)(*tensor.stride()))
        sel = Selection(ra.shape[0], ra.ctypes.data, None if keep_mask is None else keep_mask.data_ptr(),
                        None if row_index is None else row_index.data_ptr())
        xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        node = C.c_uint32()
        code = _check(lib().dmi_step_observe(self._h, point_id, C.byref(t), C.byref(sel), C.byref(xf),
                                             stream or None, C.byref(node)), allow)
        return int(node.value) if code == OK else -1

    def observe_paged(self, point_id: int, cache, block_table, reqs, *, block_size: int, n_heads: int,
                      head_dim: int, heads_sel: Sequence[int], stream: int, out_dtype: Optional[int] = None,
                      summary_mask: int = 0, keep_mask=None, allow: Sequence[int] = ()) -> int:
        dt = _torch_dtype_code(cache)
        ra = _reqs_buffer(reqs)
        kv = PagedKV(cache.data_ptr(), dt, cache.stride(0), cache.stride(1), cache.stride(2),
                     block_size, n_heads, head_dim, cache.shape[0], block_table.shape[0],
                     block_table.data_ptr(), block_table.stride(0), len(heads_sel),
                     (C.c_uint32 * 8)(*heads_sel))
        sel = Selection(ra.shape[0], ra.ctypes.data, None if keep_mask is None else keep_mask.data_ptr(), None)
        xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        node = C.c_uint32()
        code = _check(lib().dmi_step_observe_paged(self._h, point_id, C.byref(kv), C.byref(sel), C.byref(xf),
                                                   stream or None, C.byref(node)), allow)
        return int(node.value) if code == OK else -1

    def observe_batch(self, point_ids, tensors, reqs, *, stream: int, out_dtype: Optional[int] = None,
                      summary_mask: int = 0, keep_mask=None, row_index=None, paged=None,
                      allow: Sequence[int] = ()) -> int:
        """n tensors of one layout -> n consecutive records of the step, one launch.
        Returns the index of the first record, or -1 if every point is disabled."""
        tensors = list(tensors)
        _same_layout(tensors)
        n, t0 = len(tensors), tensors[0]
        dt = _torch_dtype_code(t0)
        ra = _reqs_buffer(reqs)
        pts = (C.c_uint32 * n)(*[int(p) for p in point_ids])
        data = (C.c_void_p * n)(*[t.data_ptr() for t in tensors])
        sel = Selection(ra.shape[0], ra.ctypes.data, None if keep_mask is None else keep_mask.data_ptr(),
                        None if row_index is None else row_index.data_ptr())
        xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        node = C.c_uint32()
        if paged is None:
            like = Tensor(t0.data_ptr(), dt, (C.c_int64 * 2)(*t0.shape), (C.c_int64 * 2)(*t0.stride()))
            code = lib().dmi_step_observe_batch(self._h, n, pts, data, C.byref(like), C.byref(sel), C.byref(xf),
                                                stream or None, C.byref(node))
        else:
            like = _paged_struct(t0, paged)
            code = lib().dmi_step_observe_paged_batch(self._h, n, pts, data, C.byref(like), C.byref(sel),
                                                      C.byref(xf), stream or None, C.byref(node))
        _check(code, allow)
        return int(node.value) if code == OK else -1

    def seal(self):
        _check(lib().dmi_step_seal(self._h))

    def update(self, node: int, reqs, allow: Sequence[int] = ()) -> int:
        ra = _reqs_buffer(reqs)
        return _check(lib().dmi_step_update(self._h, node, ra.ctypes.data, ra.shape[0]), allow)

    def begin(self, step_id: int, stream: int, allow: Sequence[int] = ()) -> int:
        return _check(lib().dmi_step_begin(self._h, step_id, stream or None), allow)

    def end(self, stream: int) -> int:
        return _check(lib().dmi_step_end(self._h, stream or None))


class Ring:
    """Thin object wrapper: one method per C entry point."""

    def __init__(self, device_ring_bytes: int, host_ring_bytes: int, *, device_id: int = 0,
                 flags: int = 0, max_reqs_per_observe: int = 0, rank_tag: int = 0,
                 bg_min_bytes: int = 0, bg_timeout_us: int = 0, block_timeout_ms: int = 0,
                 bg_min_records: int = 0, bg_occupancy_pct: int = 0):
        cfg = RingConfig(device_ring_bytes, host_ring_bytes, device_id, flags, max_reqs_per_observe,
                         rank_tag, bg_min_bytes, bg_timeout_us, block_timeout_ms, bg_min_records,
                         bg_occupancy_pct)
        h = C.c_void_p()
        _check(lib().dmi_ring_create(C.byref(cfg), C.byref(h)))
        self._h = h
        self._views = (RecordViewC * 256)()

    # -- lifetime --------------------------------------------------------
    def destroy(self):
        if self._h:
            _check(lib().dmi_ring_destroy(self._h))
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- producer --------------------------------------------------------
    def observe(self, point_id: int, data_ptr: int, dtype: int, shape, stride, reqs, *,
                step_id: int, stream: int = 0, out_dtype: int = DT_BF16, summary_mask: int = 0,
                keep_mask_dev: int = 0, row_index_dev: int = 0, allow: Sequence[int] = ()) -> int:
        ra = _reqs_buffer(reqs)
        t = Tensor(data_ptr, dtype, (C.c_int64 * 2)(*shape), (C.c_int64 * 2)(*stride))
        sel = Selection(ra.shape[0], ra.ctypes.data, keep_mask_dev or None, row_index_dev or None)
        xf = Transform(out_dtype, summary_mask)
        return _check(lib().dmi_observe(self._h, point_id, C.byref(t), C.byref(sel), C.byref(xf),
                                        step_id, stream or None), allow)

    def observe_tensor(self, point_id: int, tensor, reqs, *, step_id: int, stream: int = 0,
                       out_dtype: Optional[int] = None, summary_mask: int = 0, keep_mask=None,
                       row_index=None, allow: Sequence[int] = ()) -> int:
        """Convenience for torch tensors on the GPU (device memory and streams only)."""
        dt = _torch_dtype_code(tensor)
        return self.observe(point_id, tensor.data_ptr(), dt, tuple(tensor.shape),
                            tuple(tensor.stride()), reqs, step_id=step_id, stream=stream,
                            out_dtype=dt if out_dtype is None else out_dtype,
                            summary_mask=summary_mask,
                            keep_mask_dev=0 if keep_mask is None else keep_mask.data_ptr(),
                            row_index_dev=0 if row_index is None else row_index.data_ptr(),
                            allow=allow)

    def observe_paged(self, point_id: int, cache, block_table, reqs, *, block_size: int,
                      n_heads: int, head_dim: int, heads_sel: Sequence[int], step_id: int,
                      stream: int = 0, out_dtype: Optional[int] = None, summary_mask: int = 0,
                      keep_mask=None, allow: Sequence[int] = ()) -> int:
        """cache: torch tensor [blocks, slots, heads, dim]; block_table: int32 [n_seqs, max_blocks]."""
        dt = _torch_dtype_code(cache)
        ra = _reqs_buffer(reqs)
        kv = PagedKV(cache.data_ptr(), dt, cache.stride(0), cache.stride(1), cache.stride(2),
                     block_size, n_heads, head_dim, cache.shape[0], block_table.shape[0],
                     block_table.data_ptr(), block_table.stride(0), len(heads_sel),
                     (C.c_uint32 * 8)(*heads_sel))
        sel = Selection(ra.shape[0], ra.ctypes.data,
                        None if keep_mask is None else keep_mask.data_ptr(), None)
        xf = Transform(dt if out_dtype is None else out_dtype, summary_mask)
        return _check(lib().dmi_observe_paged(self._h, point_id, C.byref(kv), C.byref(sel),
                                              C.byref(xf), step_id, stream or None), allow)

    def observe_batch(self, point_ids, tensors, reqs, *, step_id: int, stream: int = 0,
                      out_dtype: Optional[int] = None, summary_mask: int = 0, keep_mask=None, row_index=None,
                      paged=None, allow: Sequence[int] = ()):
        """dmi_observe_batch / dmi_observe_paged_batch (paged: an object with block_table, block_size,
        n_heads, head_dim, heads_sel; tensors are then the caches).  Returns (status, n_done)."""
        po = PreparedBatch(self, point_ids, tensors, reqs, out_dtype=out_dtype, summary_mask=summary_mask,
                           keep_mask=keep_mask, row_index=row_index, paged=paged)
        rc, done = po(step_id, stream or None)
        _check(rc, allow)
        return rc, done

    # -- consumer --------------------------------------------------------
    def drain(self, flags: int = 0, allow: Sequence[int] = ()) -> int:
        moved = C.c_uint64()
        code = _check(lib().dmi_drain(self._h, flags, C.byref(moved)), allow)
        self.last_drain_status = code
        return int(moved.value)

    def poll_host(self, max_records: int = 256) -> List[RecordView]:
        n = C.c_uint32()
        m = min(max_records, len(self._views))
        _check(lib().dmi_poll_host(self._h, self._views, m, C.byref(n)))
        return [RecordView(v.seq, v.p0 or 0, v.n0, v.p1 or 0, v.n1) for v in self._views[: n.value]]

    def poll_host_raw(self, max_records: int = 256):
        """As poll_host, without building Python objects: (n, ctypes array of views)."""
        n = C.c_uint32()
        _check(lib().dmi_poll_host(self._h, self._views, min(max_records, len(self._views)), C.byref(n)))
        return n.value, self._views

    def release_host(self, upto_seq: int):
        _check(lib().dmi_release_host(self._h, upto_seq))

    # -- policy / stats --------------------------------------------------
    def set_policy(self, mode: int, sample_k: int = 1, sample_phase: int = 0):
        p = Policy(mode, sample_k, sample_phase)
        _check(lib().dmi_set_policy(self._h, C.byref(p)))

    def point_enable(self, point_id: int, enabled: bool):
        _check(lib().dmi_point_enable(self._h, point_id, int(enabled)))

    def get_stats(self) -> Stats:
        s = StatsC()
        _check(lib().dmi_get_stats(self._h, C.byref(s)))
        return Stats(**{n: int(getattr(s, n)) for n in _STAT_FIELDS})

    def get_point_drops(self, point_id: int) -> int:
        n = C.c_uint64()
        _check(lib().dmi_get_point_drops(self._h, point_id, C.byref(n)))
        return int(n.value)

    def free_bytes(self) -> int:
        n = C.c_uint64()
        _check(lib().dmi_ring_free_bytes(self._h, C.byref(n)))
        return int(n.value)

    def set_keep_mask(self, keep, stream: int = 0) -> int:
        """Upload a keep vector; returns the device address to pass as keep_mask_dev."""
        k = np.ascontiguousarray(np.asarray(keep, dtype=np.uint8))
        out = C.c_void_p()
        _check(lib().dmi_set_keep_mask(self._h, k.ctypes.data if k.size else None, k.size, stream or None,
                                       C.byref(out)))
        return int(out.value or 0)

    # -- exporter stages 2-3 -----------------------------------------------
    def exporter_start(self, max_pageable_bytes: int, n_copy_threads: int = 0):
        _check(lib().dmi_exporter_start(self._h, max_pageable_bytes, n_copy_threads))

    def exporter_next(self, timeout_ms: int = 100) -> Optional["SliceC"]:
        """The next per-request slice, or None after timeout_ms.  Release it when done."""
        sl = SliceC()
        rc = _check(lib().dmi_exporter_next(self._h, C.byref(sl), timeout_ms), allow=(ERR_AGAIN,))
        return None if rc == ERR_AGAIN else sl

    def exporter_next_many(self, buf, timeout_ms: int = 100) -> int:
        """Fill a (SliceC * n) array with the slices ready now; returns how many."""
        n = C.c_uint32()
        _check(lib().dmi_exporter_next_many(self._h, buf, len(buf), C.byref(n), timeout_ms), allow=(ERR_AGAIN,))
        return int(n.value)

    def exporter_release_many(self, buf, n: int):
        _check(lib().dmi_exporter_release_many(self._h, buf, n))

    def exporter_release(self, sl: "SliceC"):
        _check(lib().dmi_exporter_release(self._h, C.byref(sl)))

    def exporter_stop(self):
        _check(lib().dmi_exporter_stop(self._h))

    def debug_fill_rings(self, value: int):
        _check(lib().dmi_debug_fill_rings(self._h, value))

    def debug_exporter_allocs(self):
        """(buffers taken from the allocator, records that reused an idle buffer) of the exporter's copy stage."""
        a, b = C.c_uint64(0), C.c_uint64(0)
        _check(lib().dmi_debug_exporter_allocs(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value
