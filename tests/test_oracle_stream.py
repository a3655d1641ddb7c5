"""Pins for the oracle's ring / policy model: conservation, ordering,
wrap-around, capacity independence, and a byte-level brute-force ring."""
import hashlib
import json
import os

import numpy as np
import pytest
import torch

from oracle.decode import decode_stream
from oracle.replay import run_workload
from oracle.stream import (ERR_AGAIN, ERR_TOO_LARGE, OK, POINT_DISABLED, POLICY_BLOCK,
                           POLICY_DROP_NEWEST, SAMPLED_OUT, OracleRing)
from workloads import configs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _t(T=8, E=24, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(T, E, generator=g).to(torch.bfloat16)


def test_config1_stream_size_and_golden_hash(oracle):
    """128 records of 64 + 64 + 4*256*2 = 2,176 bytes; the digest on file was
    written by tests/golden/make_golden.py, which calls only the oracle."""
    ring = run_workload(configs.config1_tiny())
    s = ring.stream()
    assert s.size == 278528 and ring.stats.captured_records == 128
    recs = decode_stream(s)
    assert [r.seq for r in recs] == list(range(128))
    assert all(r.record_bytes == 2176 and r.n_rows == 4 and r.row_elems == 256 for r in recs)
    with open(os.path.join(GOLDEN, "config1_stream.json")) as f:
        gold = json.load(f)
    assert gold["bytes"] == s.size
    assert gold["sha256"] == hashlib.sha256(s.tobytes()).hexdigest()


@pytest.mark.parametrize("dev,host", [(8192, 16384), (4096, 4096), (1 << 20, 4 << 20)])
def test_block_stream_is_independent_of_ring_capacities(oracle, dev, host):
    ref = run_workload(configs.config1_tiny()).stream()
    got = run_workload(configs.config1_tiny(), device_ring_bytes=dev, host_ring_bytes=host)
    assert np.array_equal(got.stream(), ref)
    assert got.stats.dropped_records == 0 and got.drained == ref.size


def test_per_point_step_order_and_row_conservation(oracle):
    wl = configs.config1_tiny()
    wl.policy_mode, wl.sample_k = POLICY_DROP_NEWEST, 2
    ring = run_workload(wl, device_ring_bytes=4352, drain_every=2)   # room for two records
    recs = decode_stream(ring.stream())
    st = ring.stats
    selected = 8 * 16 * 4
    assert sum(r.n_rows for r in recs) + st.dropped_rows + st.sampled_out_rows == selected
    assert st.sampled_out_calls == 64 and st.dropped_records > 0
    assert st.captured_records + st.dropped_records == ring.next_seq
    last = {}
    for r in recs:
        assert r.step_id % 2 == 0
        assert last.get(r.point_id, -1) <= r.step_id
        last[r.point_id] = r.step_id
    present = {r.seq for r in recs}
    assert present.isdisjoint(ring.dropped_seqs)
    assert present | set(ring.dropped_seqs) == set(range(ring.next_seq))
    assert sum(st.point_drops.values()) == st.dropped_records


def test_status_codes_and_counters(oracle):
    ring = OracleRing(4096, 8192, POLICY_BLOCK)
    t = _t()
    kw = dict(out_dtype=1)
    ring.point_enable(3, False)
    assert ring.observe(t, [(0, 0, 0, 2, 1)], point_id=3, step_id=0, **kw) == POINT_DISABLED
    ring.set_policy(POLICY_BLOCK, 4, 1)
    assert ring.observe(t, [(0, 0, 0, 2, 1)], point_id=1, step_id=0, **kw) == SAMPLED_OUT
    assert ring.observe(t, [(0, 0, 0, 2, 1)], point_id=1, step_id=5, **kw) == OK
    assert ring.next_seq == 1 and ring.stats.sampled_out_rows == 2 and ring.stats.disabled_calls == 1
    big = _t(200, 24)
    assert ring.observe(big, [(0, 0, 0, 200, 1)], point_id=1, step_id=5, **kw) == ERR_TOO_LARGE
    assert ring.next_seq == 1
    # host ring full and never released: the completeness policy cannot make room
    ring = OracleRing(1024, 1024, POLICY_BLOCK)
    rc = [ring.observe(t, [(0, 0, 0, 8, 1)], point_id=0, step_id=s, **kw) for s in range(6)]
    # record = 64 + 64 + 384 = 512 bytes: two fill the device ring, the flush moves them to
    # the host ring, two more fill the device ring again, then nothing can move
    assert rc == [OK, OK, OK, OK, ERR_AGAIN, ERR_AGAIN] and ring.next_seq == 4


class _ByteRing:
    """Brute force: physical rings as byte arrays with a per-byte 'live' flag;
    any overwrite of a live byte or read of a dead one is an error."""

    def __init__(self, dev_cap, host_cap):
        self.dev = np.zeros(dev_cap, np.uint8)
        self.dev_live = np.zeros(dev_cap, bool)
        self.host = np.zeros(host_cap, np.uint8)
        self.host_live = np.zeros(host_cap, bool)
        self.head = self.tail = self.hhead = self.htail = 0
        self.out = []

    def dev_free(self):
        return int((~self.dev_live).sum())

    def write(self, rec):
        for b in rec:
            i = self.head % self.dev.size
            assert not self.dev_live[i]
            self.dev[i], self.dev_live[i] = b, True
            self.head += 1

    def drain(self):
        n = 0
        while self.tail < self.head and not self.host_live[self.hhead % self.host.size]:
            i, j = self.tail % self.dev.size, self.hhead % self.host.size
            assert self.dev_live[i]
            self.host[j], self.host_live[j] = self.dev[i], True
            self.dev_live[i] = False
            self.tail += 1
            self.hhead += 1
            n += 1
        return n

    def release(self, nbytes):
        for _ in range(nbytes):
            j = self.htail % self.host.size
            assert self.host_live[j]
            self.out.append(self.host[j])
            self.host_live[j] = False
            self.htail += 1


@pytest.mark.parametrize("seed", range(6))
def test_drop_policy_against_byte_level_brute_force(oracle, seed):
    rng = np.random.default_rng(seed)
    dev_cap, host_cap = 1024, 1536
    ring = OracleRing(dev_cap, host_cap, POLICY_DROP_NEWEST)
    brute = _ByteRing(dev_cap, host_cap)
    t = _t(8, 24, seed)
    expect_drop = []
    for op in range(10):
        rows = int(rng.integers(0, 9))
        before = ring.stats.dropped_records
        rc = ring.observe(t, [(op, 0, 0, rows, 1)], point_id=op % 3, step_id=op, out_dtype=1)
        assert rc == OK
        size = oracle.record_bytes(1, rows, 24, 1, 0)
        if size <= brute.dev_free():
            assert ring.stats.dropped_records == before
            brute.write(ring.records[-1])
        else:
            assert ring.stats.dropped_records == before + 1
            expect_drop.append(op)
        if rng.random() < 0.4:
            assert ring.drain() == brute.drain()
            if rng.random() < 0.7:
                seqs = ring.polled_seqs()
                if seqs:
                    r0 = ring.released
                    ring.release(seqs[-1])
                    brute.release(ring.released - r0)
    assert ring.dropped_seqs == expect_drop
    while ring.drained < ring.appended:
        assert ring.drain() == brute.drain()
        seqs = ring.polled_seqs()
        r0 = ring.released
        ring.release(seqs[-1])
        brute.release(ring.released - r0)
    assert np.array_equal(np.array(brute.out, np.uint8), ring.stream())


def test_host_ring_image_wraps_bytewise(oracle):
    ring = run_workload(configs.config1_tiny(n_points=2, n_steps=3), host_ring_bytes=4096,
                        device_ring_bytes=4352)
    s = ring.stream()
    img = ring.host_ring_image()
    assert s.size == 6 * 2176 > 4096
    for b in range(s.size - 4096, s.size):
        assert img[b % 4096] == s[b]


def test_replay_cache_never_hands_out_another_objects_host_copy():
    """The replay driver caches host copies per object; a short-lived object's address may
    be reused by the next one, which must not get the earlier one's copy."""
    import gc
    import torch
    from oracle.replay import CpuView
    from workloads.configs import PagedSpec
    view = CpuView()
    for k in range(50):
        table = torch.full((2, 3), k, dtype=torch.int32)
        spec = PagedSpec(16, 4, 64, [1], table)
        assert int(view.paged(spec).block_table[0, 0]) == k
        del spec, table
        gc.collect()
