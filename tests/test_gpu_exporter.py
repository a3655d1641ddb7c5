"""Exporter stages 2-3 (pinned -> pageable copy, reconstruct, slice by request)
against the oracle's independent decoder."""
import ctypes

import numpy as np
import pytest
import torch

from oracle.decode import decode_stream
from oracle.replay import run_workload
from workloads import configs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
_ELEM = {0: 0, 1: 2, 2: 2, 3: 4, 4: 1}
_NP = {1: np.uint16, 2: np.uint16, 3: np.float32, 4: np.uint8}


def _arr(ptr, n, dtype):
    if not ptr or n == 0:
        return None
    nbytes = n * np.dtype(dtype).itemsize
    return np.frombuffer((ctypes.c_uint8 * nbytes).from_address(ptr), dtype=dtype).copy()


@pytest.mark.parametrize("which", ["tiny", "decode_summaries", "paged"])
def test_slices_equal_the_decoders(which):
    from paper_2605_11093_amd import binding as B
    from paper_2605_11093_amd.replay import observe_call
    if which == "tiny":
        wl = configs.config1_tiny(device=DEV)
    elif which == "decode_summaries":
        wl = configs.config2_decode8b(device=DEV, n_points=3, n_steps=4, hidden=1024, n_reqs=16)
    else:
        wl = configs.config4_paged_kv(device=DEV, n_layers_cap=1, n_blocks=512, n_reqs=8, ctx_lo=20, ctx_hi=300,
                                      reqs_per_step=3, n_steps=3)
    expect = []
    for rec in decode_stream(run_workload(wl).stream()):
        for q in range(rec.n_reqs):
            if rec.req_table[q, 3]:
                off = int(rec.req_table[:q, 3].sum())
                n = int(rec.req_table[q, 3])
                expect.append((rec.seq, q, rec, off, n))
    got = []
    # a small pageable budget and a small host ring: the exporter has to recycle both
    with B.Ring(1 << 20, 1 << 20, flags=B.BG_THREAD, block_timeout_ms=5000) as ring:
        ring.exporter_start(1 << 19)
        s = torch.cuda.current_stream()
        with pytest.raises(B.DmiError):
            ring.poll_host()                    # the exporter is the only consumer now

        def take(limit):
            while len(got) < limit:
                sl = ring.exporter_next(2000)
                assert sl is not None, "exporter produced no slice in 2 s"
                es = _ELEM[sl.out_dtype]
                rows = _arr(sl.rows, sl.n_rows * sl.row_elems, _NP[sl.out_dtype]) if es else None
                got.append(dict(seq=sl.seq, step=sl.step_id, point=sl.point_id, q=sl.req_index, req_id=sl.req_id,
                                tok_start=sl.tok_start, tok_step=sl.tok_step, n_rows=sl.n_rows,
                                row_elems=sl.row_elems, out_dtype=sl.out_dtype, rows=rows,
                                l2=_arr(sl.l2, sl.n_rows, np.float32), mean=_arr(sl.mean, sl.n_rows, np.float32),
                                absmax=_arr(sl.absmax, sl.n_rows, np.float32)))
                ring.exporter_release(sl)

        issued = 0
        for step, calls in wl.steps():
            for c in calls:
                observe_call(ring, c, s.cuda_stream, [])
                issued += 1
            take(min(len(expect), len(got) + 4))        # consume while producing
        take(len(expect))
        assert ring.exporter_next(50) is None
        ring.exporter_stop()
        s.synchronize()
        st = ring.get_stats()
        assert st.dropped_records == 0 and st.released_bytes == st.captured_bytes
        allocated, reused = ring.debug_exporter_allocs()       # pageable buffers are pooled, not allocated per record
        assert allocated + reused == st.captured_records       # (the reuse rate itself is checked on the CPU build)
    assert len(got) == len(expect)
    for g, (seq, q, rec, off, n) in zip(got, expect):
        assert (g["seq"], g["q"], g["step"], g["point"]) == (seq, q, rec.step_id, rec.point_id)
        assert (g["req_id"], g["tok_start"], g["tok_step"], g["n_rows"]) == tuple(int(x) for x in rec.req_table[q])
        assert g["row_elems"] == rec.row_elems and g["out_dtype"] == rec.out_dtype
        if rec.out_dtype:
            assert np.array_equal(g["rows"].reshape(n, rec.row_elems), rec.payload[off:off + n])
        for bit, key in ((1, "l2"), (2, "mean"), (4, "absmax")):
            if bit in rec.summaries:
                ref = rec.summaries[bit][off:off + n]
                assert np.allclose(g[key], ref, rtol=1e-3, atol=1e-5), key
            else:
                assert g[key] is None
