"""Backpressure policies, hook filtering, error paths and the asynchronous mode,
through the C ABI on the GPU, held against the oracle's ring model."""
import numpy as np
import pytest
import torch

import oracle as orc
from oracle.decode import decode_record, record_offsets
from oracle.replay import CpuView, observe_call as oracle_observe
from oracle.stream import OracleRing, POLICY_BLOCK, POLICY_DROP_NEWEST
from workloads import configs, prng

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


def _t(rows=64, E=256, seed=1):
    return prng.randn_bf16(prng.sub_seed(21, seed), rows * E, DEV).view(rows, E)


def _reqs(n, rows_each=1):
    return np.array([(100 + i, i * rows_each, 0, rows_each, 1) for i in range(n)], dtype=np.uint32)


def test_disabled_point_and_sampling_take_no_sequence_number(B):
    t = _t()
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream().cuda_stream
        ring.point_enable(7, False)
        assert ring.observe_tensor(7, t, _reqs(4), step_id=0, stream=s) == B.POINT_DISABLED
        ring.set_policy(B.POLICY_BLOCK, 4, 1)
        assert ring.observe_tensor(1, t, _reqs(4), step_id=0, stream=s) == B.SAMPLED_OUT
        assert ring.observe_tensor(1, t, _reqs(4), step_id=5, stream=s) == B.OK
        ring.point_enable(7, True)
        assert ring.observe_tensor(7, t, _reqs(2), step_id=9, stream=s) == B.OK
        ring.drain(B.DRAIN_FLUSH)
        v = ring.poll_host()
        assert [x.seq for x in v] == [0, 1]
        assert decode_record(v[0].bytes()).step_id == 5 and decode_record(v[1].bytes()).point_id == 7
        st = ring.get_stats()
        assert (st.observed_calls, st.disabled_calls, st.sampled_out_calls, st.sampled_out_rows) == (4, 1, 1, 4)
        assert st.launched_records == 2 and st.captured_records == 2 and st.captured_rows == 6


def test_too_large_and_invalid_arguments(B):
    t = _t(64, 256)
    with B.Ring(8192, 8192) as ring:
        s = torch.cuda.current_stream().cuda_stream
        with pytest.raises(B.DmiError) as e:
            ring.observe_tensor(0, t, _reqs(32), step_id=0, stream=s)     # 64+512+16384 bytes
        assert e.value.code == B.ERR_TOO_LARGE
        for bad in ([(1, 60, 0, 5, 1)], [(1, 0, 63, 2, 1)], [(1, 0, 0, 3, 32)]):
            with pytest.raises(B.DmiError) as e:
                ring.observe_tensor(0, t, np.array(bad, np.uint32), step_id=0, stream=s)
            assert e.value.code == B.ERR_INVALID_ARG
        with pytest.raises(B.DmiError) as e:
            ring.observe_tensor(0, t.float(), _reqs(1), step_id=0, stream=s, out_dtype=B.DT_FP8)
        assert e.value.code == B.ERR_INVALID_ARG
        with pytest.raises(B.DmiError):
            ring.observe_tensor(5000, t, _reqs(1), step_id=0, stream=s)
        assert ring.get_stats().launched_records == 0
        assert ring.observe_tensor(0, t, _reqs(8), step_id=0, stream=s) == B.OK
        ring.drain(B.DRAIN_FLUSH)
        assert len(ring.poll_host()) == 1


def test_block_returns_again_when_the_host_ring_is_never_released(B):
    t = _t(8, 192)          # record = 64 + 128 + 8*384 = 3264 bytes; rings of 6400 hold one whole record
    ref = OracleRing(6400, 6400, POLICY_BLOCK)
    with B.Ring(6400, 6400, block_timeout_ms=30) as ring:
        s = torch.cuda.current_stream().cuda_stream
        rcs, want = [], []
        for step in range(6):
            rcs.append(ring.observe_tensor(0, t, _reqs(8), step_id=step, stream=s, allow=(B.ERR_AGAIN,)))
            want.append(ref.observe(t.cpu(), _reqs(8), point_id=0, step_id=step, out_dtype=1))
        assert rcs == want
        assert want == [0, 0, 0, B.ERR_AGAIN, B.ERR_AGAIN, B.ERR_AGAIN]
        assert ring.get_stats().launched_records == ref.next_seq == 3
        v = ring.poll_host()
        assert [x.seq for x in v] == ref.polled_seqs() == [0]
        ring.release_host(0)
        ref.release(0)
        assert ring.observe_tensor(0, t, _reqs(8), step_id=6, stream=s) == B.OK
        assert ref.observe(t.cpu(), _reqs(8), point_id=0, step_id=6, out_dtype=1) == 0
        torch.cuda.current_stream().synchronize()
        ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
        ref.drain()
        assert ring.last_drain_status == B.ERR_AGAIN and ref.drained < ref.appended
        got = [x.seq for x in ring.poll_host()]
        assert got == ref.polled_seqs() and got


def test_drop_newest_lockstep_counts_and_point_drops(B):
    t = _t(16, 256)         # 16 rows: record = 64 + 256 + 8192 = 8512 bytes
    dev_cap = 8512 * 3 + 64
    ref = OracleRing(dev_cap, 1 << 20, POLICY_DROP_NEWEST)
    with B.Ring(dev_cap, 1 << 20) as ring:
        ring.set_policy(B.POLICY_DROP_NEWEST)
        s = torch.cuda.current_stream()
        for step in range(4):
            for p in range(3):
                ring.observe_tensor(p, t, _reqs(16), step_id=step, stream=s.cuda_stream)
                ref.observe(t.cpu(), _reqs(16), point_id=p, step_id=step, out_dtype=1)
            if step % 2 == 1:
                ring.drain(B.DRAIN_FLUSH)
                ref.drain()
        ring.drain(B.DRAIN_FLUSH)
        ref.drain()
        got = np.concatenate([v.bytes() for v in ring.poll_host()])
        assert np.array_equal(got, ref.stream())
        st = ring.get_stats()
        assert st.dropped_records == ref.stats.dropped_records == 6
        assert st.dropped_rows == ref.stats.dropped_rows and st.dropped_bytes == ref.stats.dropped_bytes
        for p in range(3):
            assert ring.get_point_drops(p) == ref.stats.point_drops.get(p, 0)


@pytest.mark.parametrize("mode", ["copy", "kernel"])
def test_async_drop_newest_with_background_drain_keeps_the_invariants(B, mode):
    """Which records drop is timing dependent; what must hold: every record present is the
    oracle's record of that seq, seqs increase, gaps are exactly the counted drops."""
    wl = configs.config5_saturation(device=DEV, n_points=6, n_steps=12, hidden=2048, n_reqs=64)
    flags = B.BG_THREAD | (B.DRAIN_KERNEL if mode == "kernel" else 0)
    expected, sizes, rows = {}, {}, {}
    view = CpuView()
    oref = OracleRing(1 << 30, 1 << 30, POLICY_BLOCK)
    got = []
    with B.Ring(1 << 20, 1 << 22, flags=flags, bg_min_bytes=4096, bg_timeout_us=50) as ring:
        ring.set_policy(B.POLICY_DROP_NEWEST)
        s = torch.cuda.current_stream()
        from paper_2605_11093_amd.replay import observe_call
        for step, calls in wl.steps():
            for c in calls:
                observe_call(ring, c, s.cuda_stream, [])
                oracle_observe(oref, c, view)
            for v in ring.poll_host():
                got.append((v.seq, v.bytes()))
                ring.release_host(v.seq)
        s.synchronize()
        for _ in range(200):
            ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
            vs = ring.poll_host()
            for v in vs:
                got.append((v.seq, v.bytes()))
                ring.release_host(v.seq)
            if ring.last_drain_status == B.OK and not vs:
                break
        st = ring.get_stats()
    ref_recs = {int(r[8:16].view(np.uint64)[0]): r for r in oref.records}
    seqs = [q for q, _ in got]
    assert seqs == sorted(set(seqs))
    for q, b in got:
        assert np.array_equal(b, ref_recs[q]), q
    missing = sorted(set(ref_recs) - set(seqs))
    assert len(missing) == st.dropped_records
    assert sum(ref_recs[q].size for q in missing) == st.dropped_bytes
    assert sum(int(ref_recs[q][36:40].view(np.uint32)[0]) for q in missing) == st.dropped_rows
    assert st.captured_records + st.dropped_records == st.launched_records == len(ref_recs)


def test_async_block_with_background_drain_loses_nothing(B):
    from paper_2605_11093_amd.replay import run_workload_gpu
    from oracle.replay import run_workload
    wl = configs.config2_decode8b(device=DEV, n_points=4, n_steps=12, hidden=1024, n_reqs=32,
                                  device_ring_bytes=256 << 10, host_ring_bytes=512 << 10)
    got = run_workload_gpu(wl, flags=B.BG_THREAD, lockstep=False, poison=0xA5)
    from _util import compare_streams
    compare_streams(got.stream, run_workload(wl).stream())
    assert got.stats.dropped_records == 0


def test_two_rings_do_not_interact(B):
    t1, t2 = _t(32, 256, 1), _t(32, 256, 2)
    with B.Ring(1 << 20, 1 << 20, rank_tag=1) as r1, B.Ring(1 << 20, 1 << 20, rank_tag=2) as r2:
        s = torch.cuda.current_stream().cuda_stream
        for step in range(3):
            r1.observe_tensor(0, t1, _reqs(5), step_id=step, stream=s)
            r2.observe_tensor(0, t2, _reqs(7), step_id=step, stream=s)
        r1.drain(B.DRAIN_FLUSH)
        r2.drain(B.DRAIN_FLUSH)
        a, b = r1.poll_host(), r2.poll_host()
        assert [v.seq for v in a] == [0, 1, 2] == [v.seq for v in b]
        for step in range(3):
            assert np.array_equal(a[step].bytes(), orc.build_record(t1.cpu(), _reqs(5), seq=step, step_id=step,
                                                                    point_id=0, out_dtype=1, rank_tag=1))
            assert np.array_equal(b[step].bytes(), orc.build_record(t2.cpu(), _reqs(7), seq=step, step_id=step,
                                                                    point_id=0, out_dtype=1, rank_tag=2))


def test_record_straddling_the_host_ring_end_comes_back_in_two_spans(B):
    t = _t(16, 256)         # 8512-byte records into a 20,480-byte host ring
    with B.Ring(1 << 16, 20480) as ring:
        s = torch.cuda.current_stream().cuda_stream
        out = []
        for step in range(7):
            ring.observe_tensor(0, t, _reqs(16), step_id=step, stream=s)
            ring.drain(B.DRAIN_FLUSH)
            for v in ring.poll_host():
                out.append((v.n1 > 0, v.bytes()))
                ring.release_host(v.seq)
        assert any(two for two, _ in out) and len(out) == 7
        for step, (_, b) in enumerate(out):
            assert np.array_equal(b, orc.build_record(t.cpu(), _reqs(16), seq=step, step_id=step, point_id=0,
                                                      out_dtype=1))


@pytest.mark.parametrize("flags_name", ["none", "bg"])
def test_commit_accounting_across_policy_and_mask_changes(B, flags_name):
    """How the host learns what was committed differs by launch kind (sizes known on the
    host under the completeness policy without a keep vector; read back from the device
    otherwise).  A sequence that keeps switching kinds, with drains in between, must
    still add up: same stream, same counters as the oracle."""
    from workloads import prng as P
    t = _t(64, 256, seed=9)
    tc = t.cpu()
    flags = B.BG_THREAD if flags_name == "bg" else 0
    ref = OracleRing(8 << 20, 32 << 20, POLICY_BLOCK)
    kinds = P.randint(P.sub_seed(77, 1), 150, 0, 2)
    sizes = P.randint(P.sub_seed(77, 2), 150, 1, 20)
    drains = P.randint(P.sub_seed(77, 3), 150, 0, 6)
    keep_alive = []
    with B.Ring(8 << 20, 32 << 20, flags=flags, bg_min_bytes=4096) as ring:
        s = torch.cuda.current_stream()
        got = []
        for i in range(150):
            kind, n = int(kinds[i]), int(sizes[i])
            reqs = np.array([(i * 100 + r, 3 * r, 0, 1 + (r + i) % 3, 1) for r in range(n)], dtype=np.uint32)
            keep = None
            if kind == 1:       # completeness policy, keep vector: sizes decided on the device
                keep = (P.randint(P.sub_seed(77, 4, i), n, 0, 1)).astype(np.uint8)
            mode = B.POLICY_DROP_NEWEST if kind == 2 else B.POLICY_BLOCK
            ring.set_policy(mode)
            ref.mode = POLICY_DROP_NEWEST if kind == 2 else POLICY_BLOCK
            km = None
            if keep is not None and i % 2:
                km = torch.from_numpy(keep).to(DEV)     # caller-owned: the host cannot tell the record's size
                keep_alive.append(km)
            elif keep is not None:
                class _Ptr:                             # library-owned: the host kept a copy and can
                    p = ring.set_keep_mask(keep, s.cuda_stream)

                    def data_ptr(self):
                        return self.p
                km = _Ptr()
            assert ring.observe_tensor(i % 7, t, reqs, step_id=i, stream=s.cuda_stream, keep_mask=km,
                                       summary_mask=i % 8) == B.OK
            assert ref.observe(tc, reqs, point_id=i % 7, step_id=i, out_dtype=1, summary_mask=i % 8,
                               keep_mask=keep) == 0
            if drains[i] == 0:
                ring.drain(0)               # moves what has committed by now, whatever that is
                for v in ring.poll_host():
                    got.append(v.bytes())
                    ring.release_host(v.seq)
        s.synchronize()
        ring.drain(B.DRAIN_FLUSH)
        for v in ring.poll_host():
            got.append(v.bytes())
        ref.drain()
        from _util import compare_streams
        compare_streams(np.concatenate(got), ref.stream())
        st = ring.get_stats()
        assert (st.captured_records, st.captured_rows, st.captured_bytes, st.dropped_records) == \
            (ref.stats.captured_records, ref.stats.captured_rows, ref.stats.captured_bytes, 0)


def test_flush_waits_for_batches_the_drain_thread_issued(B):
    """dmi_drain(FLUSH) returning DMI_OK means every record captured so far can be polled,
    also when the library's drain thread issued the last copy while the flush was waiting
    for an earlier one."""
    wl = configs.config2_decode8b(device=DEV, n_points=16, n_steps=4)
    calls = [wl.step_calls(s) for s in range(4)]
    from paper_2605_11093_amd import PreparedObserve
    with B.Ring(256 << 20, 1 << 30, flags=B.BG_THREAD, max_reqs_per_observe=256, block_timeout_ms=2000) as ring:
        s = torch.cuda.current_stream()
        pos = [[PreparedObserve(ring, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype, summary_mask=c.summary_mask)
                for c in calls[k]] for k in range(4)]

        def consume():
            while True:
                k, views = ring.poll_host_raw()
                if not k:
                    return
                ring.release_host(views[k - 1].seq)

        for trial in range(12):
            for step in range(48):
                for po in pos[step % 4]:
                    assert po(step, s.cuda_stream) == B.OK
                consume()
            s.synchronize()
            while True:
                ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
                consume()
                if ring.last_drain_status == B.OK:
                    break
            st = ring.get_stats()
            assert st.released_bytes == st.captured_bytes == st.drained_bytes, (trial, st)


def test_nonblocking_drain_on_a_ring_with_a_drain_thread_becomes_visible(B):
    """A caller's non-blocking drain on a ring whose drain thread is running: nothing else is
    pending afterwards, and still the copies it issued must be noted as finished (by the drain
    thread) so that the records can be polled."""
    import time
    t = prng.randn_bf16(61, 64 * 1024, DEV).view(64, 1024)
    reqs = np.array([(i, i, 0, 1, 1) for i in range(64)], dtype=np.uint32)
    # thresholds the drain thread will not reach by itself for a long time
    with B.Ring(1 << 22, 1 << 22, flags=B.BG_THREAD, bg_min_bytes=1 << 21, bg_timeout_us=5_000_000) as ring:
        s = torch.cuda.current_stream()
        ring.observe_tensor(0, t, reqs, step_id=0, stream=s.cuda_stream)
        s.synchronize()
        moved = 0
        for _ in range(2000):                      # the commit has to be noticed first
            moved += ring.drain(B.DRAIN_NONBLOCK)
            if moved:
                break
            time.sleep(0.001)
        assert moved == orc.record_bytes(64, 64, 1024, 1, 0)
        views = []
        for _ in range(2000):
            views = ring.poll_host()
            if views:
                break
            time.sleep(0.001)
        assert len(views) == 1 and views[0].seq == 0
        ref = orc.build_record(t.cpu(), reqs, seq=0, step_id=0, point_id=0, out_dtype=1)
        assert np.array_equal(views[0].bytes(), ref)


def test_a_record_larger_than_the_host_ring_is_refused(B):
    t = prng.randn_bf16(62, 64 * 1024, DEV).view(64, 1024)
    reqs = np.array([(0, 0, 0, 64, 1)], dtype=np.uint32)          # 128 KiB of payload
    with B.Ring(1 << 20, 1 << 16) as ring:                        # device ring 1 MiB, host ring 64 KiB
        rc = ring.observe_tensor(0, t, reqs, step_id=0, allow=(B.ERR_TOO_LARGE,))
        assert rc == B.ERR_TOO_LARGE
        assert ring.get_stats().launched_records == 0
        ring.observe_tensor(0, t, np.array([(0, 0, 0, 16, 1)], dtype=np.uint32), step_id=0)   # 32 KiB fits
        ring.drain(B.DRAIN_FLUSH)
        assert len(ring.poll_host()) == 1


OFF64, OFF32 = (1 << 64) - 1, (1 << 32) - 1


@pytest.mark.parametrize("trigger", ["bytes", "records", "occupancy", "timeout"])
def test_each_drain_threshold_alone_starts_a_batch(B, trigger):
    """The drain thread's four batching thresholds (ready entries, occupancy, byte count, timeout):
    with three of them switched off, the fourth alone must start a batch once it is reached, and
    nothing may be drained before."""
    import time
    t = prng.randn_bf16(63, 64 * 1024, DEV).view(64, 1024)
    one = np.array([(0, 0, 0, 1, 1)], dtype=np.uint32)             # 64 + 64 + 2048 = 2176 bytes
    many = np.array([(0, 0, 0, 40, 1)], dtype=np.uint32)           # 64 + 64 + 81920 = 82048 bytes
    kw = dict(bg_min_bytes=OFF64, bg_min_records=OFF32, bg_occupancy_pct=101, bg_timeout_us=OFF32)
    if trigger == "bytes":
        kw["bg_min_bytes"], below, reach = 100_000, (many, 1), (many, 1)        # 82 KB, then 164 KB
    elif trigger == "records":
        kw["bg_min_records"], below, reach = 5, (one, 4), (one, 1)
    elif trigger == "occupancy":
        kw["bg_occupancy_pct"], below, reach = 25, (many, 3), (many, 1)          # 1 MiB ring: 246 KB, then 328 KB
    else:
        kw["bg_timeout_us"], below, reach = 30_000, None, (one, 1)
    with B.Ring(1 << 20, 1 << 22, flags=B.BG_THREAD, **kw) as ring:
        s = torch.cuda.current_stream()

        def settle_commits():
            s.synchronize()
            time.sleep(0.02)            # the drain thread notices the commits (its probe comes after 200 us of quiet)

        n_rec = 0
        if below is not None:
            for _ in range(below[1]):
                ring.observe_tensor(0, t, below[0], step_id=0, stream=s.cuda_stream)
                n_rec += 1
            settle_commits()
            st = ring.get_stats()
            assert st.captured_records == n_rec and st.drain_batches == 0 and st.drained_bytes == 0
        t0 = time.monotonic()
        for _ in range(reach[1]):
            ring.observe_tensor(0, t, reach[0], step_id=0, stream=s.cuda_stream)
            n_rec += 1
        s.synchronize()
        if trigger == "timeout":
            time.sleep(0.005)
            assert ring.get_stats().drain_batches == 0              # 5 ms in: not yet
        for _ in range(2000):
            st = ring.get_stats()
            if st.drain_batches:
                break
            time.sleep(0.001)
        assert st.drain_batches >= 1 and st.drained_bytes == st.captured_bytes and st.captured_records == n_rec
        if trigger == "timeout":
            assert time.monotonic() - t0 >= 0.030
        for _ in range(200):
            if len(ring.poll_host()) or ring.get_stats().released_bytes:
                break
            time.sleep(0.001)
