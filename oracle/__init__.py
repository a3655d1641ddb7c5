"""CPU oracle for the capture-and-stage path -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares nothing with the HIP library: the arithmetic lives in
dmi_oracle.c (plain C, gcc), the ring/policy model in stream.py, and an
independent record decoder in decode.py.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None

DT_NONE, DT_BF16, DT_FP16, DT_FP32, DT_FP8 = 0, 1, 2, 3, 4
_TORCH_DT = {torch.bfloat16: DT_BF16, torch.float16: DT_FP16, torch.float32: DT_FP32}


def build(force: bool = False) -> str:
    """Compile dmi_oracle.c with gcc (building the checker is not using it)."""
    src = os.path.join(_HERE, "dmi_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


class _Req(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("req_id", "row_base", "tok_start", "tok_count", "tok_step")]


class _Dense(C.Structure):
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_uint32), ("n_rows", C.c_int64),
                ("row_elems", C.c_int64), ("row_stride", C.c_int64)]


class _Paged(C.Structure):
    _fields_ = [("base", C.c_void_p), ("dtype", C.c_uint32), ("block_stride", C.c_int64),
                ("slot_stride", C.c_int64), ("head_stride", C.c_int64),
                ("block_size", C.c_uint32), ("n_heads", C.c_uint32), ("head_dim", C.c_uint32),
                ("block_table", C.c_void_p), ("block_table_stride", C.c_int64),
                ("n_heads_sel", C.c_uint32), ("heads_sel", C.c_uint32 * 8)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = C.CDLL(_SO)
        L.orc_bf16_value.restype = C.c_double
        L.orc_bf16_value.argtypes = [C.c_uint16]
        L.orc_fp16_value.restype = C.c_double
        L.orc_fp16_value.argtypes = [C.c_uint16]
        L.orc_fp8_value.restype = C.c_double
        L.orc_fp8_value.argtypes = [C.c_uint8]
        L.orc_bf16_to_fp8.restype = C.c_uint8
        L.orc_bf16_to_fp8.argtypes = [C.c_uint16]
        L.orc_bf16_to_fp16.restype = C.c_uint16
        L.orc_bf16_to_fp16.argtypes = [C.c_uint16]
        L.orc_record_bytes.restype = C.c_uint64
        L.orc_record_bytes.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_build_dense.restype = C.c_int64
        L.orc_build_dense.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32,
                                      C.c_uint32, C.POINTER(_Dense), C.c_void_p, C.c_uint32,
                                      C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32]
        L.orc_build_paged.restype = C.c_int64
        L.orc_build_paged.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32,
                                      C.c_uint32, C.POINTER(_Paged), C.c_void_p, C.c_uint32,
                                      C.c_void_p, C.c_uint32, C.c_uint32]
        _lib = L
    return _lib


def bf16_to_fp8(bits: int) -> int:
    return lib().orc_bf16_to_fp8(bits)


def bf16_to_fp16(bits: int) -> int:
    return lib().orc_bf16_to_fp16(bits)


def fp8_value(code: int) -> float:
    return lib().orc_fp8_value(code)


def fp16_value(code: int) -> float:
    return lib().orc_fp16_value(code)


def record_bytes(n_reqs, n_rows, row_elems, out_dtype, summary_mask) -> int:
    return int(lib().orc_record_bytes(n_reqs, n_rows, row_elems, out_dtype, summary_mask))


def _reqs_array(reqs) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
    return a


def build_record(tensor: torch.Tensor, reqs, *, seq: int, step_id: int, point_id: int,
                 out_dtype: int, summary_mask: int = 0, keep_mask=None, row_index=None,
                 paged=None, rank_tag: int = 0) -> np.ndarray:
    """One record's bytes (uint8 array).

    tensor: CPU tensor.  dense -> [T, E] with stride[1] == 1; paged -> the cache
    [blocks, slots, heads, dim] with `paged` an object carrying block_size,
    n_heads, head_dim, heads_sel and a CPU int32 block_table [n_seqs, max_blocks].
    """
    assert tensor.device.type == "cpu"
    L = lib()
    ra = _reqs_array(reqs)
    n_reqs = ra.shape[0]
    km = None if keep_mask is None else np.ascontiguousarray(np.asarray(keep_mask, dtype=np.uint8))
    ri = None if row_index is None else np.ascontiguousarray(np.asarray(row_index, dtype=np.int32))
    kept = ra[:, 3].astype(np.int64) * (1 if km is None else (km != 0))
    n_rows = int(kept.sum())
    src_dt = _TORCH_DT[tensor.dtype]
    if paged is None:
        assert tensor.dim() == 2 and (tensor.shape[1] <= 1 or tensor.stride(1) == 1)
        row_elems = tensor.shape[1]
    else:
        row_elems = len(paged.heads_sel) * paged.head_dim
    size = record_bytes(n_reqs, n_rows, row_elems, out_dtype, summary_mask)
    out = np.empty(size, dtype=np.uint8)
    kmp = km.ctypes.data if km is not None else None
    rip = ri.ctypes.data if ri is not None else None
    if paged is None:
        d = _Dense(tensor.data_ptr(), src_dt, tensor.shape[0], tensor.shape[1], tensor.stride(0))
        n = L.orc_build_dense(out.ctypes.data, size, seq, step_id, point_id, rank_tag, C.byref(d),
                              ra.ctypes.data, n_reqs, kmp, rip, out_dtype, summary_mask)
    else:
        bt = paged.block_table
        assert bt.device.type == "cpu" and bt.dtype == torch.int32 and bt.stride(1) == 1
        assert tensor.dim() == 4 and tensor.stride(3) == 1
        p = _Paged(tensor.data_ptr(), src_dt, tensor.stride(0), tensor.stride(1), tensor.stride(2),
                   paged.block_size, paged.n_heads, paged.head_dim, bt.data_ptr(), bt.stride(0),
                   len(paged.heads_sel), (C.c_uint32 * 8)(*paged.heads_sel))
        n = L.orc_build_paged(out.ctypes.data, size, seq, step_id, point_id, rank_tag, C.byref(p),
                              ra.ctypes.data, n_reqs, kmp, out_dtype, summary_mask)
    if n != size:
        raise ValueError(f"oracle record build failed: code {n} (expected size {size})")
    return out
