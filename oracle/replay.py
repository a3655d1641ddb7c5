"""Drive a synthetic workload through the oracle's ring model -- TEST
INFRASTRUCTURE ONLY.  The workload object is duck-typed (steps() yielding
(step, calls); each call has tensor / reqs / point_id / step_id / out_dtype /
summary_mask / keep_mask / row_index / paged attributes)."""
from __future__ import annotations

import torch

from .stream import OracleRing


class _CpuPaged:
    def __init__(self, p):
        self.block_size, self.n_heads, self.head_dim = p.block_size, p.n_heads, p.head_dim
        self.heads_sel = list(p.heads_sel)
        self.block_table = p.block_table.cpu().contiguous()


class CpuView:
    """Host copies of a workload's device tensors, made once per tensor."""

    def __init__(self):
        self._t, self._p = {}, {}

    def tensor(self, t: torch.Tensor) -> torch.Tensor:
        if t.device.type == "cpu":
            return t
        # the cache keeps the original alive: a key made of an address must not outlive its object
        key = (t.data_ptr(), tuple(t.shape), tuple(t.stride()))
        if key not in self._t:
            self._t[key] = (t, t.cpu())
        return self._t[key][1]

    def paged(self, p):
        if p is None:
            return None
        if id(p) not in self._p:
            self._p[id(p)] = (p, _CpuPaged(p))
        return self._p[id(p)][1]


def observe_call(ring: OracleRing, call, view: CpuView) -> int:
    return ring.observe(view.tensor(call.tensor), call.reqs, point_id=call.point_id,
                        step_id=call.step_id, out_dtype=call.out_dtype,
                        summary_mask=call.summary_mask, keep_mask=call.keep_mask,
                        row_index=call.row_index, paged=view.paged(call.paged))


def run_workload(wl, *, drain_every: int = 1, release: bool = True, keep_records: bool = True,
                 device_ring_bytes=None, host_ring_bytes=None, max_steps=None) -> OracleRing:
    """Lockstep schedule: all of a step's observes, then (every `drain_every`
    steps) one drain followed by release of everything polled."""
    ring = OracleRing(device_ring_bytes or wl.device_ring_bytes,
                      host_ring_bytes or wl.host_ring_bytes,
                      wl.policy_mode, wl.sample_k, 0, keep_records=keep_records)
    view = CpuView()
    for step, calls in wl.steps():
        if max_steps is not None and step >= max_steps:
            break
        for c in calls:
            rc = observe_call(ring, c, view)
            if rc == -5 and release:
                # completeness policy with a full host ring: the consumer frees what it
                # has polled, then the producer's flush can proceed
                seqs = ring.polled_seqs()
                if seqs:
                    ring.release(seqs[-1])
                rc = observe_call(ring, c, view)
            if rc < 0:
                raise RuntimeError(f"oracle observe failed with {rc} at step {step} point {c.point_id}")
        if (step + 1) % drain_every == 0:
            ring.drain()
            if release:
                seqs = ring.polled_seqs()
                if seqs:
                    ring.release(seqs[-1])
    while ring.drained < ring.appended:
        if ring.drain() == 0:
            break
        if release:
            seqs = ring.polled_seqs()
            if seqs:
                ring.release(seqs[-1])
    return ring
