"""Pins for the oracle's record builder: gathers, paged gathers, summaries and
layout, each against something other than the builder itself."""
import numpy as np
import pytest
import torch

from oracle.decode import decode_record, decode_stream

DT_NONE, DT_BF16, DT_FP16, DT_FP32, DT_FP8 = 0, 1, 2, 3, 4


def _counter_tensor(T, E, dtype=torch.bfloat16, pad=0):
    """Every element a distinct, exactly representable value (needs T*E <= 256
    for bf16 beyond integers up to 256; use int16 view instead)."""
    base = torch.arange(T * (E + pad), dtype=torch.int32).to(torch.int16)
    t = base.view(torch.bfloat16) if dtype == torch.bfloat16 else base.view(torch.float16)
    return t.view(T, E + pad)[:, :E]


def _bits(t):
    return t.contiguous().view(torch.int16).numpy().astype(np.uint16)


def test_all_rows_one_request_is_memcpy(oracle):
    t = _counter_tensor(13, 40)
    rec = oracle.build_record(t, [(7, 0, 0, 13, 1)], seq=3, step_id=9, point_id=2, out_dtype=DT_BF16)
    r = decode_record(rec)
    assert r.n_rows == 13 and r.row_elems == 40 and r.seq == 3 and r.step_id == 9 and r.point_id == 2
    assert rec[64 + 64: 64 + 64 + 13 * 40 * 2].tobytes() == t.contiguous().view(torch.int16).numpy().tobytes()
    assert rec.size == 64 + 64 + 1088      # 1040 payload bytes padded to 1088
    assert oracle.record_bytes(1, 13, 40, DT_BF16, 0) == rec.size


@pytest.mark.parametrize("E", [1, 2, 7, 8, 33, 40])
@pytest.mark.parametrize("pad", [0, 3])
def test_ragged_gather_equals_index_select(oracle, E, pad):
    """Second route: numpy fancy indexing on the same bytes."""
    T = 50
    t = _counter_tensor(T, E, pad=pad)
    reqs = [(100, 0, 2, 3, 1), (101, 10, 0, 5, 4), (102, 40, 9, 1, 1), (103, 45, 0, 0, 1)]
    rows = [0 + 2 + j for j in range(3)] + [10 + 4 * j for j in range(5)] + [49]
    rec = oracle.build_record(t, reqs, seq=0, step_id=0, point_id=0, out_dtype=DT_BF16)
    r = decode_record(rec)
    assert (r.payload == _bits(t)[rows]).all()
    assert (r.req_table == np.array([[100, 2, 1, 3], [101, 0, 4, 5], [102, 9, 1, 1], [103, 0, 1, 0]])).all()
    assert r.flags == 0
    # unique counters: every payload element decodes back to (row, col)
    stride = E + pad
    vals = r.payload.astype(np.int64)
    assert (vals // stride == np.array(rows)[:, None]).all()
    assert (vals % stride == np.arange(E)[None, :]).all()


def test_keep_mask_compacts_and_zeroes_counts(oracle):
    t = _counter_tensor(30, 8)
    reqs = [(1, 0, 0, 2, 1), (2, 5, 0, 3, 1), (3, 10, 1, 2, 2), (4, 20, 0, 1, 1)]
    rec = oracle.build_record(t, reqs, seq=0, step_id=0, point_id=0, out_dtype=DT_BF16,
                              keep_mask=[1, 0, 1, 0])
    r = decode_record(rec)
    assert r.flags == 2 and r.n_rows == 4
    assert (r.req_table[:, 3] == [2, 0, 2, 0]).all()
    assert (r.payload == _bits(t)[[0, 1, 11, 13]]).all()
    assert (r.rows_of(2) == _bits(t)[[11, 13]]).all()
    # all-dropped mask: header + table only
    rec0 = oracle.build_record(t, reqs, seq=0, step_id=0, point_id=0, out_dtype=DT_BF16,
                               keep_mask=[0, 0, 0, 0])
    assert rec0.size == 128 and decode_record(rec0).n_rows == 0


def test_explicit_row_index_mode(oracle):
    t = _counter_tensor(30, 8)
    reqs = [(1, 0, 77, 2, 1), (2, 0, 5, 3, 9)]
    idx = [29, 3, 7, 7, 0]
    r = decode_record(oracle.build_record(t, reqs, seq=0, step_id=0, point_id=0,
                                          out_dtype=DT_BF16, row_index=idx))
    assert r.flags == 4 and (r.payload == _bits(t)[idx]).all()
    # masked-out requests still consume their listed rows
    r = decode_record(oracle.build_record(t, reqs, seq=0, step_id=0, point_id=0,
                                          out_dtype=DT_BF16, row_index=idx, keep_mask=[0, 1]))
    assert r.flags == 6 and (r.payload == _bits(t)[[7, 7, 0]]).all()


def test_out_of_range_selection_is_refused(oracle):
    t = _counter_tensor(4, 8)
    with pytest.raises(ValueError):
        oracle.build_record(t, [(1, 3, 0, 2, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_BF16)


class _Paged:
    def __init__(self, bs, nh, hd, sel, table):
        self.block_size, self.n_heads, self.head_dim, self.heads_sel = bs, nh, hd, sel
        self.block_table = torch.tensor(table, dtype=torch.int32)


def test_paged_gather_decodes_to_block_slot_head_dim(oracle):
    """Element value encodes (block, slot, head, dim); the payload must list
    exactly the addressed ones in (request, token, selected head, dim) order."""
    NB, BS, NH, HD = 12, 4, 3, 8
    n = NB * BS * NH * HD
    cache = torch.arange(n, dtype=torch.int32).to(torch.int16).view(torch.bfloat16).view(NB, BS, NH, HD)
    table = [[5, 2, 9, 0], [11, 7, 3, 1]]
    spec = _Paged(BS, NH, HD, [2, 0], table)
    reqs = [(50, 1, 3, 6, 1), (51, 0, 0, 4, 3)]      # row_base = row of the block table
    r = decode_record(oracle.build_record(cache, reqs, seq=0, step_id=0, point_id=0,
                                          out_dtype=DT_BF16, paged=spec))
    assert r.flags == 1 and r.row_elems == 16 and r.n_rows == 10
    toks = [(1, 3 + j) for j in range(6)] + [(0, 3 * j) for j in range(4)]
    for g, (seq_row, t) in enumerate(toks):
        blk, slot = table[seq_row][t // BS], t % BS
        for k, h in enumerate([2, 0]):
            want = ((blk * BS + slot) * NH + h) * HD + np.arange(HD)
            assert (r.payload[g, k * HD:(k + 1) * HD].astype(np.int64) == want).all()


def test_paged_with_identity_table_reduces_to_dense(oracle):
    NB, BS, NH, HD = 6, 4, 1, 8
    cache = _counter_tensor(NB * BS, HD).contiguous().view(NB, BS, NH, HD)
    spec = _Paged(BS, NH, HD, [0], [list(range(NB))])
    reqs_p = [(9, 0, 2, 7, 3)]
    a = decode_record(oracle.build_record(cache, reqs_p, seq=0, step_id=0, point_id=0,
                                          out_dtype=DT_BF16, paged=spec))
    b = decode_record(oracle.build_record(cache.view(NB * BS, HD), [(9, 0, 2, 7, 3)], seq=0,
                                          step_id=0, point_id=0, out_dtype=DT_BF16))
    assert (a.payload == b.payload).all()


def _f32(x):
    return np.float32(x)


def test_summaries_closed_forms(oracle):
    E = 96
    rows = torch.zeros(5, E, dtype=torch.bfloat16)
    rows[0, :] = -1.5                                    # constant c: L2 |c| sqrt(E), mean c, absmax |c|
    rows[1, 17] = 3.0                                    # one-hot
    rows[2, 0::2] = 1.0
    rows[2, 1::2] = -1.0                                 # alternating: mean 0, L2 sqrt(E)
    rows[3, :] = torch.arange(E).to(torch.bfloat16)      # 0..95 exact in bf16
    r = decode_record(oracle.build_record(rows, [(0, 0, 0, 5, 1)], seq=0, step_id=0, point_id=0,
                                          out_dtype=DT_NONE, summary_mask=7))
    assert r.payload_bytes == 0 and r.record_bytes == 64 + 64 + 3 * 64
    l2, mean, amax = r.summaries[1], r.summaries[2], r.summaries[4]
    assert l2[0] == _f32(1.5 * np.sqrt(96.0)) and mean[0] == _f32(-1.5) and amax[0] == _f32(1.5)
    assert l2[1] == 3.0 and mean[1] == _f32(3.0 / 96) and amax[1] == 3.0
    assert l2[2] == _f32(np.sqrt(96.0)) and mean[2] == 0.0 and amax[2] == 1.0
    n = 95
    assert l2[3] == _f32(np.sqrt(n * (n + 1) * (2 * n + 1) / 6.0)) and mean[3] == _f32(n / 2.0) and amax[3] == 95.0
    assert l2[4] == 0 and mean[4] == 0 and amax[4] == 0


def test_summaries_second_route_numpy_float64_and_nan_inf(oracle):
    g = torch.Generator().manual_seed(5)
    x = torch.randn(9, 333, generator=g).to(torch.bfloat16)
    x[7, 5] = float("inf")
    x[8, 6] = float("nan")
    for dt in (torch.bfloat16, torch.float16, torch.float32):
        xs = x.to(dt)
        r = decode_record(oracle.build_record(xs, [(0, 0, 0, 9, 1)], seq=0, step_id=0, point_id=0,
                                              out_dtype=DT_NONE, summary_mask=5))
        v = xs.double().numpy()
        with np.errstate(invalid="ignore", over="ignore"):
            assert np.array_equal(r.summaries[1][:7], np.sqrt((v[:7] ** 2).sum(1)).astype(np.float32))
            assert np.array_equal(r.summaries[4][:7], np.abs(v[:7]).max(1).astype(np.float32))
        assert np.isinf(r.summaries[1][7]) and np.isinf(r.summaries[4][7])
        assert np.isnan(r.summaries[1][8]) and np.isnan(r.summaries[4][8])
        assert 2 not in r.summaries


def test_downcast_payload_equals_torch_cast(oracle):
    g = torch.Generator().manual_seed(11)
    x = (torch.randn(6, 64, generator=g) * 3).to(torch.bfloat16)
    r8 = decode_record(oracle.build_record(x, [(0, 0, 0, 6, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_FP8))
    r16 = decode_record(oracle.build_record(x, [(0, 0, 0, 6, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_FP16))
    assert (r8.payload == x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()).all()
    assert (r16.payload == _bits(x.to(torch.float16))).all()
    assert r8.payload_bytes == 6 * 64 and r16.payload_bytes == 6 * 64 * 2


def test_raw_copy_of_fp32_and_fp16_sources(oracle):
    x = torch.arange(24, dtype=torch.float32).view(3, 8) * 0.37
    r = decode_record(oracle.build_record(x, [(0, 1, 0, 2, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_FP32))
    assert np.array_equal(r.payload, x[1:3].numpy()) and r.src_dtype == 3
    h = x.to(torch.float16)
    r = decode_record(oracle.build_record(h, [(0, 0, 0, 3, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_FP16))
    assert (r.payload == _bits(h)).all()
    with pytest.raises(ValueError):       # downcasts are defined from bf16 only
        oracle.build_record(x, [(0, 0, 0, 1, 1)], seq=0, step_id=0, point_id=0, out_dtype=DT_FP8)


def test_layout_invariants_over_random_shapes(oracle):
    rng = np.random.default_rng(0)
    for _ in range(60):
        T, E = int(rng.integers(1, 30)), int(rng.integers(1, 70))
        n_reqs = int(rng.integers(0, 6))
        reqs = []
        for q in range(n_reqs):
            base = int(rng.integers(0, T))
            cnt = int(rng.integers(0, T - base + 1))
            reqs.append((q, base, 0, cnt, 1))
        out_dt = int(rng.choice([DT_NONE, DT_BF16, DT_FP16, DT_FP8]))
        sm = int(rng.integers(0, 8))
        km = None if rng.random() < 0.5 else rng.integers(0, 2, n_reqs).astype(np.uint8)
        t = _counter_tensor(T, E)
        rec = oracle.build_record(t, np.array(reqs, dtype=np.uint32).reshape(-1, 5), seq=5, step_id=6,
                                  point_id=7, out_dtype=out_dt, summary_mask=sm, keep_mask=km, rank_tag=3)
        r = decode_record(rec)          # raises on any inconsistency or non-zero pad
        assert r.record_bytes == rec.size and r.rank_tag == 3 and rec.size % 64 == 0
        kept = sum(c[3] for i, c in enumerate(reqs) if km is None or km[i])
        assert r.n_rows == kept
        assert oracle.record_bytes(n_reqs, kept, E, out_dt, sm) == rec.size
