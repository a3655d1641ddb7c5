"""Ring / policy model of the oracle -- TEST INFRASTRUCTURE ONLY.

The captured data forms one logical byte stream: the records of all admitted
observations, in hook-execution order (paper section 4.2: ring entries are in
FIFO order aligned with hook execution).  A physical ring of capacity C holds
stream byte b at offset b mod C, so the stream does not depend on either ring's
capacity as long as nothing is dropped.

Policies (paper section 4.4, plus this build's readings):
  * completeness ("block"): nothing is lost; when the incoming record does not
    fit the device ring the producer first has the ring flushed.
  * best effort, record granular ("drop-newest"): an incoming record that does
    not fit the free space of the device ring is discarded whole and counted.
  * 1-in-k step sampling: an observation is taken only if step_id % k == phase;
    others take no sequence number and are counted apart from drops.
  * hook filtering: a disabled point is the identity; no record, no sequence
    number.

This model is *lockstep*: every call completes before the next one starts, and
bytes move from the device ring to the host ring only inside drain().

Pins (tests/test_oracle_stream.py): a separate byte-level brute-force simulation of
the drop policy on small random schedules; ring-capacity independence of the stream
under the completeness policy; row conservation (captured + dropped + sampled-out =
listed); per-point step order; the configuration-1 stream's size and SHA-256
(tests/golden, written by make_golden.py from this package alone).  Parity unpinned:
the readings themselves (what drop-newest discards, where block waits, what 1-in-k
counts) are this build's where the paper is silent; the tests pin the model to those
readings, not the readings to the paper.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import build_record, record_bytes

OK, SAMPLED_OUT, POINT_DISABLED = 0, 1, 2
ERR_TOO_LARGE, ERR_AGAIN = -3, -5
POLICY_BLOCK, POLICY_DROP_NEWEST = 0, 1


@dataclass
class Stats:
    observed_calls: int = 0
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
    point_drops: dict = field(default_factory=dict)


class OracleRing:
    def __init__(self, device_ring_bytes: int, host_ring_bytes: int, policy_mode: int = 0,
                 sample_k: int = 1, sample_phase: int = 0, rank_tag: int = 0,
                 keep_records: bool = True):
        assert device_ring_bytes % 64 == 0 and host_ring_bytes % 64 == 0
        self.dev_cap, self.host_cap = device_ring_bytes, host_ring_bytes
        self.mode, self.k, self.phase = policy_mode, sample_k, sample_phase
        self.rank_tag = rank_tag
        self.keep_records = keep_records
        self.next_seq = 0
        self.appended = 0      # stream bytes written into the device ring so far
        self.drained = 0       # stream bytes moved on to the host ring
        self.released = 0      # stream bytes the consumer has given back
        self.records: List[np.ndarray] = []      # admitted records, in order
        self.spans: List[tuple] = []             # (seq, start, end) per admitted record
        self.dropped_seqs: List[int] = []
        self.disabled = set()
        self.stats = Stats()

    # -- control ---------------------------------------------------------
    def set_policy(self, mode: int, sample_k: int = 1, sample_phase: int = 0):
        assert sample_k >= 1 and 0 <= sample_phase < sample_k
        self.mode, self.k, self.phase = mode, sample_k, sample_phase

    def point_enable(self, point_id: int, enabled: bool):
        (self.disabled.discard if enabled else self.disabled.add)(point_id)

    # -- producer --------------------------------------------------------
    def observe(self, tensor, reqs, *, point_id: int, step_id: int, out_dtype: int,
                summary_mask: int = 0, keep_mask=None, row_index=None, paged=None) -> int:
        st = self.stats
        st.observed_calls += 1
        ra = np.asarray(reqs, dtype=np.uint32).reshape(-1, 5)
        listed_rows = int(ra[:, 3].astype(np.int64).sum())
        if point_id in self.disabled:
            st.disabled_calls += 1
            return POINT_DISABLED
        if step_id % self.k != self.phase:
            st.sampled_out_calls += 1
            st.sampled_out_rows += listed_rows
            return SAMPLED_OUT
        row_elems = tensor.shape[1] if paged is None else len(paged.heads_sel) * paged.head_dim
        upper = record_bytes(ra.shape[0], listed_rows, row_elems, out_dtype, summary_mask)
        if upper > self.dev_cap:
            return ERR_TOO_LARGE
        if self.mode == POLICY_BLOCK and self.appended - self.drained + upper > self.dev_cap:
            self.drain()        # the completeness policy's flush
            if self.appended - self.drained + upper > self.dev_cap:
                return ERR_AGAIN
        seq = self.next_seq
        self.next_seq += 1
        rec = build_record(tensor, ra, seq=seq, step_id=step_id, point_id=point_id,
                           out_dtype=out_dtype, summary_mask=summary_mask, keep_mask=keep_mask,
                           row_index=row_index, paged=paged, rank_tag=self.rank_tag)
        n_rows = int(rec[36:40].view(np.uint32)[0])
        if self.mode == POLICY_DROP_NEWEST and self.appended - self.drained + rec.size > self.dev_cap:
            st.dropped_records += 1
            st.dropped_rows += n_rows
            st.dropped_bytes += rec.size
            st.point_drops[point_id] = st.point_drops.get(point_id, 0) + 1
            self.dropped_seqs.append(seq)
            return OK
        self.spans.append((seq, self.appended, self.appended + rec.size))
        self.appended += rec.size
        if self.keep_records:
            self.records.append(rec)
        st.captured_records += 1
        st.captured_rows += n_rows
        st.captured_bytes += rec.size
        return OK

    # -- consumer --------------------------------------------------------
    def drain(self) -> int:
        """Move what fits from the device ring to the host ring."""
        n = min(self.appended - self.drained, self.host_cap - (self.drained - self.released))
        self.drained += n
        self.stats.drained_bytes += n
        return n

    def polled_seqs(self) -> List[int]:
        """Sequence numbers of the records completely present in the host ring
        and not yet released."""
        return [s for (s, a, b) in self.spans if a >= self.released and b <= self.drained]

    def release(self, upto_seq: int):
        for (s, a, b) in self.spans:
            if s <= upto_seq and b <= self.drained and b > self.released:
                self.stats.released_bytes += b - self.released
                self.released = b

    # -- results ---------------------------------------------------------
    def stream(self) -> np.ndarray:
        """All admitted records concatenated (the expected host byte stream
        once everything has been drained)."""
        return np.concatenate(self.records) if self.records else np.zeros(0, np.uint8)

    def host_ring_image(self, fill: int = 0) -> np.ndarray:
        """What the physical host ring holds after the drains so far."""
        img = np.full(self.host_cap, fill, dtype=np.uint8)
        s = self.stream()[: self.drained]
        lo = max(0, self.drained - self.host_cap)
        for b0 in range(lo - lo % self.host_cap, self.drained, self.host_cap):
            a, b = max(b0, lo), min(b0 + self.host_cap, self.drained)
            img[a % self.host_cap: a % self.host_cap + (b - a)] = s[a:b]
        return img
