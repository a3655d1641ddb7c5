"""Parity at the full shapes, ring sizes and policies of the five benchmark configurations, in the launch
configuration bench.py times (asynchronous: non-blocking drains issued by the
producer thread, or the library's drain thread).  The oracle cannot build these
streams whole in seconds, so: every record's header is checked against what the
call sequence fixes (properties that hold at any size), and a spread sample of
records is compared with the oracle's record byte for byte.  Step counts are cut
where a configuration's stream would take minutes; shapes are not."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as orc
from oracle.replay import CpuView
from workloads import configs
from _util import compare_record

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


class Checker:
    """on_record callback: header facts for every record, bytes kept for a sample."""

    def __init__(self, want_seq):
        self.want = set(want_seq)
        self.meta = []           # (seq, step, point, n_rows, record_bytes)
        self.kept = {}

    def __call__(self, v):
        h = np.frombuffer((ctypes.c_uint8 * 64).from_address(v.p0), dtype=np.uint8)
        assert int(h[0:4].view(np.uint32)[0]) == 0x32494D44
        seq = int(h[8:16].view(np.uint64)[0])
        assert seq == v.seq
        rb = int(h[48:56].view(np.uint64)[0])
        assert rb == v.nbytes
        self.meta.append((seq, int(h[16:24].view(np.uint64)[0]), int(h[24:28].view(np.uint32)[0]),
                          int(h[36:40].view(np.uint32)[0]), rb))
        if seq in self.want:
            self.kept[seq] = v.bytes()


def _oracle_record(call, seq, view):
    paged = view.paged(call.paged)
    return orc.build_record(view.tensor(call.tensor), call.reqs, seq=seq, step_id=call.step_id,
                            point_id=call.point_id, out_dtype=call.out_dtype,
                            summary_mask=call.summary_mask, keep_mask=call.keep_mask,
                            row_index=call.row_index, paged=paged)


def _check(run, chk, expect_drops):
    st = run.stats
    seqs = [m[0] for m in chk.meta]
    assert seqs == sorted(set(seqs)), "sequence numbers not strictly increasing"
    assert st.launched_records == len(run.launched)
    assert st.captured_records == len(seqs) and st.captured_records + st.dropped_records == st.launched_records
    assert st.captured_bytes == sum(m[4] for m in chk.meta) == st.released_bytes
    assert st.captured_rows == sum(m[3] for m in chk.meta)
    if not expect_drops:
        assert st.dropped_records == 0 and seqs == list(range(len(run.launched)))
    for seq, step, point, n_rows, rb in chk.meta:      # header vs the call that got this seq
        c = run.launched[seq]
        assert (step, point) == (c.step_id, c.point_id)
        assert n_rows == int(c.reqs[:, 3].sum())
    missing = sorted(set(range(len(run.launched))) - set(seqs))
    assert len(missing) == st.dropped_records
    view = CpuView()
    assert chk.kept, "no sampled record survived"
    for seq, got in chk.kept.items():
        compare_record(got, _oracle_record(run.launched[seq], seq, view), what=f"seq {seq}")
    return missing


def test_config2_full_decode8b(B):
    from paper_2605_11093_amd.replay import run_workload_gpu
    wl = configs.config2_decode8b(device=DEV)                         # 32 points x 256 steps, 256 MiB / 2 GiB, block
    chk = Checker(range(0, 8192, 331))
    run = run_workload_gpu(wl, collect=False, lockstep=False, drain_flags=B.DRAIN_NONBLOCK, on_record=chk,
                           block_timeout_ms=2000)
    _check(run, chk, expect_drops=False)
    assert run.stats.captured_records == 8192 and run.stats.captured_bytes == 8192 * 525888
    assert run.stats.host_ring_high_water <= 2 << 30 and run.stats.dev_ring_high_water <= 256 << 20


def test_config3_full_ragged_prefill_fp8_drop_newest(B):
    from paper_2605_11093_amd.replay import run_workload_gpu
    wl = configs.config3_prefill(device=DEV, n_steps=4)               # full shapes, 512 MiB ring, drop-newest
    chk = Checker([0, 4, 9, 13, 21, 35])                              # residual and MLP points
    run = run_workload_gpu(wl, collect=False, lockstep=False, flags=B.BG_THREAD, on_record=chk)
    missing = _check(run, chk, expect_drops=True)
    # whatever was dropped is accounted for in rows and bytes
    rows = sum(int(run.launched[q].reqs[:, 3].sum()) for q in missing)
    assert rows == run.stats.dropped_rows
    by = sum(orc.record_bytes(32, int(run.launched[q].reqs[:, 3].sum()), run.launched[q].tensor.shape[1], 4, 0)
             for q in missing)
    assert by == run.stats.dropped_bytes


def test_config4_full_paged_kv(B):
    from paper_2605_11093_amd.replay import run_workload_gpu
    wl = configs.config4_paged_kv(device=DEV, n_steps=12)             # 8 caches of 2 GiB, 2 GiB / 8 GiB rings, block
    chk = Checker([3, 40, 77])
    run = run_workload_gpu(wl, collect=False, lockstep=False, flags=B.BG_THREAD, on_record=chk,
                           block_timeout_ms=5000)
    _check(run, chk, expect_drops=False)
    assert run.stats.captured_records == 96 and run.stats.bad_rows == 0


@pytest.mark.parametrize("k,steps", [(1, 24), (4, 48)])
def test_config5_full_saturation_with_sampling(B, k, steps):
    from paper_2605_11093_amd.replay import run_workload_gpu
    wl = configs.config5_saturation(device=DEV, n_steps=steps, sample_k=k)   # 4 GiB / 16 GiB rings, drop-newest
    chk = Checker(range(0, 80 * steps, 137))
    run = run_workload_gpu(wl, collect=False, lockstep=False, flags=B.BG_THREAD, on_record=chk)
    _check(run, chk, expect_drops=True)
    st = run.stats
    assert st.sampled_out_calls == 80 * (steps - (steps + k - 1) // k)
    assert st.launched_records == 80 * ((steps + k - 1) // k)
    # conservation: every selected row is captured, dropped or sampled out
    assert st.captured_rows + st.dropped_rows + st.sampled_out_rows == 80 * steps * 256
