"""Independent record decoder / validator -- TEST INFRASTRUCTURE ONLY.

Written against the record layout alone (numpy + struct, no call into the C
builder) so that it can check the builder's output, and later the HIP path's,
from the consumer's side: the role of the paper's exporter stage that rebuilds
tensors with shape and dtype and slices them by request and token range
(section 4.3).
"""
from __future__ import annotations

import struct
from dataclasses import dataclass
from typing import List

import numpy as np

MAGIC = 0x32494D44
_HDR = struct.Struct("<IHHQQIBBBBIIIIQQ")
_ELEM = {0: 0, 1: 2, 2: 2, 3: 4, 4: 1}
_NP = {1: np.uint16, 2: np.uint16, 3: np.float32, 4: np.uint8}   # bf16/fp16 kept as bit patterns


def _pad64(n: int) -> int:
    return (n + 63) // 64 * 64


@dataclass
class Record:
    seq: int
    step_id: int
    point_id: int
    src_dtype: int
    out_dtype: int
    summary_mask: int
    flags: int
    n_reqs: int
    n_rows: int
    row_elems: int
    rank_tag: int
    record_bytes: int
    payload_bytes: int
    req_table: np.ndarray     # uint32 [n_reqs, 4]: req_id, tok_start, tok_step, n_rows_r
    payload: np.ndarray       # [n_rows, row_elems] of the out dtype's storage type (or empty)
    summaries: dict           # bit -> float32 [n_rows]

    def rows_of(self, r: int) -> np.ndarray:
        """Payload rows of request r (the exporter's slice by request)."""
        off = int(self.req_table[:r, 3].sum())
        return self.payload[off: off + int(self.req_table[r, 3])]


def decode_record(buf: np.ndarray, offset: int = 0) -> Record:
    """Decode and validate the record that starts at buf[offset]."""
    b = memoryview(np.ascontiguousarray(buf[offset: offset + 64]))
    (magic, version, hbytes, seq, step_id, point_id, src_dt, out_dt, smask, flags, n_reqs,
     n_rows, row_elems, rank_tag, rec_bytes, payload_bytes) = _HDR.unpack(b)
    if magic != MAGIC:
        raise ValueError(f"bad magic {magic:#x} at {offset}")
    if version != 1 or hbytes != 64:
        raise ValueError("bad version / header size")
    if out_dt not in _ELEM or src_dt not in (1, 2, 3) or smask & ~7 or flags & ~7:
        raise ValueError("bad dtype / mask / flags")
    table_bytes = _pad64(n_reqs * 16)
    if payload_bytes != n_rows * row_elems * _ELEM[out_dt]:
        raise ValueError("payload_bytes inconsistent with n_rows * row_elems * elem size")
    n_sum = bin(smask).count("1")
    expect = 64 + table_bytes + _pad64(payload_bytes) + n_sum * _pad64(n_rows * 4)
    if rec_bytes != expect:
        raise ValueError(f"record_bytes {rec_bytes} != section sum {expect}")
    if offset + rec_bytes > buf.size:
        raise ValueError("record runs past the end of the buffer")
    rec = buf[offset: offset + rec_bytes]
    pos = 64
    table = rec[pos: pos + n_reqs * 16].view(np.uint32).reshape(n_reqs, 4).copy()
    if rec[pos + n_reqs * 16: pos + table_bytes].any():
        raise ValueError("non-zero pad after request table")
    if int(table[:, 3].sum()) != n_rows:
        raise ValueError("n_rows != sum of per-request row counts")
    pos += table_bytes
    if out_dt:
        payload = rec[pos: pos + payload_bytes].view(_NP[out_dt]).reshape(n_rows, row_elems).copy()
    else:
        payload = np.zeros((n_rows, 0), np.uint8)
    if rec[pos + payload_bytes: pos + _pad64(payload_bytes)].any():
        raise ValueError("non-zero pad after payload")
    pos += _pad64(payload_bytes)
    sums = {}
    for bit in (1, 2, 4):
        if smask & bit:
            sums[bit] = rec[pos: pos + n_rows * 4].view(np.float32).copy()
            if rec[pos + n_rows * 4: pos + _pad64(n_rows * 4)].any():
                raise ValueError("non-zero pad after summary array")
            pos += _pad64(n_rows * 4)
    assert pos == rec_bytes
    return Record(seq, step_id, point_id, src_dt, out_dt, smask, flags, n_reqs, n_rows, row_elems,
                  rank_tag, rec_bytes, payload_bytes, table, payload, sums)


def decode_stream(buf: np.ndarray) -> List[Record]:
    """Split a byte stream into records; the stream must be exactly a whole
    number of records with strictly increasing sequence numbers."""
    out, pos, last = [], 0, -1
    while pos < buf.size:
        r = decode_record(buf, pos)
        if r.seq <= last:
            raise ValueError("sequence numbers not strictly increasing")
        last = r.seq
        out.append(r)
        pos += r.record_bytes
    return out


def record_offsets(buf: np.ndarray):
    """(seq, offset, record_bytes) of every record, reading headers only."""
    out, pos = [], 0
    while pos < buf.size:
        magic, = struct.unpack_from("<I", buf, pos)
        if magic != MAGIC:
            raise ValueError(f"bad magic at {pos}")
        seq, = struct.unpack_from("<Q", buf, pos + 8)
        n, = struct.unpack_from("<Q", buf, pos + 48)
        out.append((seq, pos, n))
        pos += n
    return out
