"""Comparison helpers for the parity tests (oracle side only: the decoder used
here is the oracle's independent one)."""
import numpy as np

from oracle.decode import decode_record, record_offsets

L2_RTOL = 1e-3          # spec tolerance for the fp32 summaries
MEAN_RTOL, MEAN_ATOL_SCALE = 1e-3, 1e-5


def _payload_mean_abs(r):
    """mean |x| of every row, from the (oracle's) payload: the scale of the mean's absolute tolerance
    when the record carries no L2."""
    p = r.payload
    if r.out_dtype == 1:
        v = (p.astype(np.uint32) << 16).view(np.float32)
    elif r.out_dtype == 2:
        v = p.view(np.float16).astype(np.float32)
    elif r.out_dtype == 3:
        v = p
    else:
        import oracle
        table = np.array([oracle.fp8_value(c) for c in range(256)], dtype=np.float64)
        v = table[p]
    return np.nanmean(np.abs(v.astype(np.float64)), axis=1)


def compare_record(got: np.ndarray, ref: np.ndarray, what="", mean_abs=None):
    """Bit-exact on header, request table, payload and pads; summaries: absmax
    exact, L2 within rel 1e-3, mean within 1e-3*|ref| + 1e-5*mean|x| (pure relative
    error on a mean is ill-posed when the sum cancels).  mean|x| is taken from the
    caller (mean_abs, per row), else bounded by L2/sqrt(E) when the record carries an
    L2, else computed from the reference payload; a record with a mean and none of
    these cannot be judged and is an error."""
    assert got.size == ref.size, f"{what}: size {got.size} != {ref.size}"
    g, r = decode_record(got), decode_record(ref)
    if not r.summary_mask:
        if not np.array_equal(got, ref):
            d = np.flatnonzero(got != ref)
            raise AssertionError(f"{what}: {d.size} bytes differ, first {d[:8]}, last {d[-3:]} of {ref.size}")
        return
    n_sum = bin(r.summary_mask).count("1")
    sum_bytes = n_sum * ((r.n_rows * 4 + 63) // 64 * 64)
    head = r.record_bytes - sum_bytes
    if not np.array_equal(got[:head], ref[:head]):
        d = np.flatnonzero(got[:head] != ref[:head])
        raise AssertionError(f"{what}: {d.size} non-summary bytes differ, first {d[:8]}, last {d[-3:]} of {head}")
    if 4 in r.summaries:
        a, b = g.summaries[4], r.summaries[4]
        nan = np.isnan(b)
        assert np.array_equal(a[~nan], b[~nan]), f"{what}: absmax differs"
    l2_ref = None
    if 1 in r.summaries:
        a, b = g.summaries[1].astype(np.float64), r.summaries[1].astype(np.float64)
        l2_ref = b
        fin = np.isfinite(b)
        assert np.array_equal(np.isnan(a), np.isnan(b)), f"{what}: L2 NaN pattern differs"
        assert np.all(np.abs(a[fin] - b[fin]) <= L2_RTOL * np.abs(b[fin])), f"{what}: L2 out of tolerance"
        inf = np.isinf(b)
        assert np.array_equal(a[inf], b[inf]), f"{what}: L2 inf differs"
    if 2 in r.summaries:
        a, b = g.summaries[2].astype(np.float64), r.summaries[2].astype(np.float64)
        fin = np.isfinite(b)
        assert np.array_equal(np.isnan(a), np.isnan(b)), f"{what}: mean NaN pattern differs"
        if mean_abs is not None:
            scale = np.asarray(mean_abs, dtype=np.float64)[fin]
        elif l2_ref is not None:
            scale = l2_ref[fin] / np.sqrt(r.row_elems)
        elif r.out_dtype:
            scale = _payload_mean_abs(r)[fin]
        else:
            raise AssertionError(f"{what}: a mean without L2, payload or mean_abs has no tolerance scale")
        tol = MEAN_RTOL * np.abs(b[fin]) + MEAN_ATOL_SCALE * scale
        assert np.all(np.abs(a[fin] - b[fin]) <= tol), f"{what}: mean out of tolerance"


def compare_streams(got: np.ndarray, ref: np.ndarray):
    assert got.size == ref.size, f"stream size {got.size} != {ref.size}"
    go, ro = record_offsets(got), record_offsets(ref)
    assert [(s, o, n) for s, o, n in go] == [(s, o, n) for s, o, n in ro], "record boundaries differ"
    for seq, off, n in ro:
        compare_record(got[off:off + n], ref[off:off + n], what=f"seq {seq}")
