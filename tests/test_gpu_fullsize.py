"""Parity at the full shapes, ring sizes and policies of the five benchmark configurations, in the launch
configurations bench.py times (asynchronous: the library's drain thread, or non-blocking
drains issued by the producer thread; observes issued singly or batched).

Every record that reaches the host ring is compared, while the workload is still running,
with the oracle's record of the same call: byte for byte (summaries to their tolerance),
straight out of the pinned ring.  Every header is also checked against what the call
sequence fixes, and the counters against the records seen.  Where drops are possible in an
asynchronous run several outcomes are valid; the lockstep variants make the drop set unique
and compare whole streams and counters with the oracle's ring model.

Coverage of each configuration's stream (the oracle builds 0.3 to 3 GB of records per second
on one core, and a GPU test has about two minutes):
  config 2   all 256 steps, all 8,192 records (4.3 GB)
  config 3   all 8 steps, all 80 records (4.3 GB), asynchronous, singly and batched; plus 4 steps in lockstep with
             the drain withheld every other step, and 4 steps with a 256 MiB device ring
  config 4   all 128 steps, all 1,024 records (37 GB) batched; 40 steps (320 records) singly
  config 5   k = 1: all 200 steps, every record that was not dropped, batched; k = 4: all 200
             steps (50 captured: 4,000 records, 16.8 GB), singly
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle as orc
from oracle.decode import decode_record
from oracle.replay import CpuView, run_workload
from workloads import configs
from _util import compare_record, compare_streams

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


def _span(p, n):
    return np.frombuffer((ctypes.c_uint8 * n).from_address(p), dtype=np.uint8)


def _oracle_record(call, seq, view):
    paged = view.paged(call.paged)
    return orc.build_record(view.tensor(call.tensor), call.reqs, seq=seq, step_id=call.step_id,
                            point_id=call.point_id, out_dtype=call.out_dtype,
                            summary_mask=call.summary_mask, keep_mask=call.keep_mask,
                            row_index=call.row_index, paged=paged)


class Checker:
    """on_record callback: every record's header facts, and its bytes against the oracle's record
    of the call that got its sequence number, compared in place (no copy out of the ring)."""

    def __init__(self, run):
        self.run = run
        self.view = CpuView()
        self.meta = []           # (seq, step, point, n_rows, record_bytes)
        self.compared_bytes = 0

    def __call__(self, v):
        h = _span(v.p0, 64)
        assert int(h[0:4].view(np.uint32)[0]) == 0x32494D44
        seq = int(h[8:16].view(np.uint64)[0])
        assert seq == v.seq
        rb = int(h[48:56].view(np.uint64)[0])
        assert rb == v.nbytes
        self.meta.append((seq, int(h[16:24].view(np.uint64)[0]), int(h[24:28].view(np.uint32)[0]),
                          int(h[36:40].view(np.uint32)[0]), rb))
        call = self.run.launched[seq]
        ref = _oracle_record(call, seq, self.view)
        assert ref.size == rb, f"seq {seq}: {rb} bytes, oracle {ref.size}"
        if call.summary_mask:
            compare_record(v.bytes(), ref, what=f"seq {seq}")
        else:
            a = _span(v.p0, v.n0)
            same = np.array_equal(a, ref[:v.n0]) and (not v.n1 or np.array_equal(_span(v.p1, v.n1), ref[v.n0:]))
            if not same:
                compare_record(v.bytes(), ref, what=f"seq {seq}")        # says where
        self.compared_bytes += rb


def _run(B, wl, **kw):
    from paper_2605_11093_amd.replay import GpuRun, run_workload_gpu
    run = GpuRun()
    chk = Checker(run)
    run_workload_gpu(wl, collect=False, lockstep=False, on_record=chk, run=run, **kw)
    return run, chk


def _check(run, chk, expect_drops):
    st = run.stats
    seqs = [m[0] for m in chk.meta]
    assert seqs == sorted(set(seqs)), "sequence numbers not strictly increasing"
    assert st.launched_records == len(run.launched)
    assert st.captured_records == len(seqs) and st.captured_records + st.dropped_records == st.launched_records
    assert st.captured_bytes == sum(m[4] for m in chk.meta) == st.released_bytes == chk.compared_bytes
    assert st.captured_rows == sum(m[3] for m in chk.meta)
    if not expect_drops:
        assert st.dropped_records == 0 and seqs == list(range(len(run.launched)))
    for seq, step, point, n_rows, rb in chk.meta:      # header vs the call that got this seq
        c = run.launched[seq]
        assert (step, point) == (c.step_id, c.point_id)
        assert n_rows == int(c.reqs[:, 3].sum())
    missing = sorted(set(range(len(run.launched))) - set(seqs))
    assert len(missing) == st.dropped_records
    return missing


def test_config2_full_decode8b_every_record(B):
    wl = configs.config2_decode8b(device=DEV)                         # 32 points x 256 steps, 256 MiB / 2 GiB, block
    run, chk = _run(B, wl, drain_flags=B.DRAIN_NONBLOCK, block_timeout_ms=5)
    _check(run, chk, expect_drops=False)
    assert run.stats.captured_records == 8192 and run.stats.captured_bytes == 8192 * 525888
    assert run.stats.host_ring_high_water <= 2 << 30 and run.stats.dev_ring_high_water <= 256 << 20


def test_config2_full_decode8b_batched_every_record(B):
    wl = configs.config2_decode8b(device=DEV)
    run, chk = _run(B, wl, flags=B.BG_THREAD, block_timeout_ms=5, batch=32)
    _check(run, chk, expect_drops=False)
    assert run.stats.captured_records == 8192 and run.stats.captured_bytes == 8192 * 525888


def _dropped_accounting(run, missing):
    rows = sum(int(run.launched[q].reqs[:, 3].sum()) for q in missing)
    assert rows == run.stats.dropped_rows
    by = sum(orc.record_bytes(32, int(run.launched[q].reqs[:, 3].sum()), run.launched[q].tensor.shape[1], 4, 0)
             for q in missing)
    assert by == run.stats.dropped_bytes


@pytest.mark.parametrize("batch", [0, 8])
def test_config3_full_ragged_prefill_fp8_every_record(B, batch):
    """batch = 8: a step's eight residual points in one launch and its two MLP points in another, the
    launches bench.py times as config3_*_batch*."""
    wl = configs.config3_prefill(device=DEV)                          # all 8 steps, 512 MiB ring, drop-newest
    run, chk = _run(B, wl, flags=B.BG_THREAD, batch=batch)
    missing = _check(run, chk, expect_drops=True)
    _dropped_accounting(run, missing)
    assert run.stats.launched_records == 80


@pytest.mark.parametrize("variant", ["drain_withheld", "ring_256MiB"])
def test_config3_full_lockstep_drop_sets_are_the_oracles(B, variant):
    """Full shapes in lockstep, so that the set of dropped records is unique: (a) the 512 MiB ring with
    the drain withheld every other step: a step's 535.6 MB leave 1.3 MB, so the whole next step is
    dropped; (b) a 256 MiB ring drained after every step: four residual records fit, the first MLP
    record (146 MB) does not, three more residual records do, the last one and the second MLP record
    do not.  Streams, drop counters and per-point drop counts must be the oracle ring model's.
    (A 128 MiB ring cannot hold an MLP record at all: that call is refused as too large, by the
    library and by the oracle's model alike.)"""
    from paper_2605_11093_amd.replay import run_workload_gpu
    kw = dict(drain_every=2) if variant == "drain_withheld" else dict(device_ring_bytes=256 << 20)
    wl = configs.config3_prefill(device=DEV, n_steps=4)
    if variant != "drain_withheld":
        from oracle.stream import OracleRing
        mlp = [c for c in wl.step_calls(0) if c.point_id >= 100][0]
        with B.Ring(128 << 20, 1 << 26, max_reqs_per_observe=wl.max_reqs) as small:
            small.set_policy(wl.policy_mode)
            rc = small.observe_tensor(mlp.point_id, mlp.tensor, mlp.reqs, step_id=0, out_dtype=mlp.out_dtype,
                                      allow=(B.ERR_TOO_LARGE,))
            assert rc == B.ERR_TOO_LARGE and small.get_stats().launched_records == 0
        model = OracleRing(128 << 20, 1 << 26, wl.policy_mode, 1, 0)
        assert model.observe(torch.empty(0, 14336, dtype=torch.bfloat16), mlp.reqs, point_id=mlp.point_id, step_id=0,
                             out_dtype=mlp.out_dtype) == B.ERR_TOO_LARGE
    ring = B.Ring(kw.get("device_ring_bytes", wl.device_ring_bytes), wl.host_ring_bytes, max_reqs_per_observe=wl.max_reqs)
    ring.set_policy(wl.policy_mode, wl.sample_k, 0)
    got = run_workload_gpu(wl, drain_every=kw.get("drain_every", 1), ring=ring)
    drops = {p: ring.get_point_drops(p) for p in list(range(8)) + [100, 101]}
    torch.cuda.synchronize()
    ring.destroy()
    ref = run_workload(wl, **kw)
    assert ref.stats.dropped_records > 0 and ref.stats.captured_records > 0
    assert [s for s, _ in got.records] == [s for s, _, _ in ref.spans]
    for (seq, rec), want in zip(got.records, ref.records):
        assert np.array_equal(rec, want), f"seq {seq}"
    a, b = got.stats, ref.stats
    assert (a.captured_records, a.captured_rows, a.captured_bytes) == (b.captured_records, b.captured_rows, b.captured_bytes)
    assert (a.dropped_records, a.dropped_rows, a.dropped_bytes) == (b.dropped_records, b.dropped_rows, b.dropped_bytes)
    assert {p: n for p, n in drops.items() if n} == b.point_drops


@pytest.mark.parametrize("batch,steps", [(8, 128), (0, 40)])
def test_config4_full_paged_kv_every_record(B, batch, steps):
    wl = configs.config4_paged_kv(device=DEV, n_steps=steps)          # 8 caches of 2 GiB, 2 GiB / 8 GiB rings, block
    run, chk = _run(B, wl, flags=B.BG_THREAD, block_timeout_ms=5, batch=batch)
    _check(run, chk, expect_drops=False)
    assert run.stats.captured_records == 8 * steps and run.stats.bad_rows == 0


@pytest.mark.parametrize("k,steps,batch", [(1, 200, 80), (4, 200, 0)])
def test_config5_full_saturation_every_surviving_record(B, k, steps, batch):
    wl = configs.config5_saturation(device=DEV, n_steps=steps, sample_k=k)   # 4 GiB / 16 GiB rings, drop-newest
    run, chk = _run(B, wl, flags=B.BG_THREAD, batch=batch)
    _check(run, chk, expect_drops=True)
    st = run.stats
    assert st.sampled_out_calls == 80 * (steps - (steps + k - 1) // k)
    assert st.launched_records == 80 * ((steps + k - 1) // k)
    # conservation: every selected row is captured, dropped or sampled out
    assert st.captured_rows + st.dropped_rows + st.sampled_out_rows == 80 * steps * 256
