"""Feed a synthetic workload (workloads.configs) through the C ABI.

Argument marshalling and scheduling only: which observe is called when, when the
ring is drained, polled and released.  PyTorch supplies device memory and the
stream handle.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np
import torch

from . import binding as B


@dataclass
class GpuRun:
    stats: B.Stats = None
    records: List[tuple] = field(default_factory=list)     # (seq, bytes) when collecting
    n_records: int = 0
    n_bytes: int = 0
    launched: List[object] = field(default_factory=list)   # launched[seq] = the call that got that seq

    @property
    def stream(self) -> np.ndarray:
        return (np.concatenate([b for _, b in self.records]) if self.records
                else np.zeros(0, np.uint8))


def observe_call(ring: B.Ring, call, stream_handle: int, keep_alive: list, allow=()) -> int:
    dev = call.tensor.device
    km = ri = None
    if call.keep_mask is not None:
        km = torch.from_numpy(np.ascontiguousarray(call.keep_mask, dtype=np.uint8)).to(dev)
        keep_alive.append(km)
    if call.row_index is not None:
        ri = torch.from_numpy(np.ascontiguousarray(call.row_index, dtype=np.int32)).to(dev)
        keep_alive.append(ri)
    if call.paged is None:
        return ring.observe_tensor(call.point_id, call.tensor, call.reqs, step_id=call.step_id,
                                   stream=stream_handle, out_dtype=call.out_dtype,
                                   summary_mask=call.summary_mask, keep_mask=km, row_index=ri,
                                   allow=allow)
    p = call.paged
    return ring.observe_paged(call.point_id, call.tensor, p.block_table, call.reqs,
                              block_size=p.block_size, n_heads=p.n_heads, head_dim=p.head_dim,
                              heads_sel=p.heads_sel, step_id=call.step_id, stream=stream_handle,
                              out_dtype=call.out_dtype, summary_mask=call.summary_mask,
                              keep_mask=km, allow=allow)


def consume(ring: B.Ring, run: GpuRun, collect: bool, release: bool,
            on_record: Optional[Callable] = None):
    """Poll every complete record, hand it on, release it."""
    while True:
        views = ring.poll_host()
        if not views:
            return
        for v in views:
            run.n_records += 1
            run.n_bytes += v.nbytes
            if collect:
                run.records.append((v.seq, v.bytes()))
            if on_record is not None:
                on_record(v)
        if release:
            ring.release_host(views[-1].seq)
        else:
            return


def run_workload_gpu(wl, *, drain_every: int = 1, release: bool = True, collect: bool = True,
                     flags: int = 0, device_ring_bytes=None, host_ring_bytes=None,
                     max_steps=None, lockstep: bool = True, on_record=None,
                     block_timeout_ms: int = 1, poison: Optional[int] = None,
                     ring: Optional[B.Ring] = None, drain_flags: int = 0,
                     bg_min_bytes: int = 0, before_observe: Optional[Callable] = None) -> GpuRun:
    """Lockstep schedule (the one the oracle's model follows): a step's observes,
    then every `drain_every` steps a flush-drain followed by poll + release.
    With lockstep=False the drain after a step moves only what has committed by
    then, without waiting for the step's kernels."""
    own = ring is None
    if own:
        ring = B.Ring(device_ring_bytes or wl.device_ring_bytes, host_ring_bytes or wl.host_ring_bytes,
                      flags=flags, max_reqs_per_observe=wl.max_reqs, block_timeout_ms=block_timeout_ms,
                      bg_min_bytes=bg_min_bytes)
        ring.set_policy(wl.policy_mode, wl.sample_k, 0)
    if poison is not None:
        ring.debug_fill_rings(poison)
    run = GpuRun()
    s = torch.cuda.current_stream()
    keep_alive: list = []
    try:
        for step, calls in wl.steps():
            if max_steps is not None and step >= max_steps:
                break
            for c in calls:
                if before_observe is not None:
                    before_observe(c, s.cuda_stream)       # e.g. the model compute that produces the tensor
                rc = observe_call(ring, c, s.cuda_stream, keep_alive, allow=(B.ERR_AGAIN,))
                tries = 0
                while rc == B.ERR_AGAIN:
                    # completeness policy, no room: this thread is also the consumer, so
                    # consume what has arrived and try again
                    consume(ring, run, collect, release, on_record)
                    tries += 1
                    rc = observe_call(ring, c, s.cuda_stream, keep_alive,
                                      allow=(B.ERR_AGAIN,) if tries < 200000 else ())
                if rc == B.OK:
                    run.launched.append(c)
            if (step + 1) % drain_every == 0:
                if lockstep:
                    s.synchronize()     # every kernel of the step has committed
                ring.drain(B.DRAIN_FLUSH if lockstep else drain_flags, allow=(B.ERR_AGAIN,))
                consume(ring, run, collect, release, on_record)
                keep_alive.clear() if lockstep else None
        # tail: everything still in flight
        s.synchronize()
        deadline = time.monotonic() + 60.0
        while True:
            if time.monotonic() > deadline:
                raise RuntimeError("final drain made no progress for 60 s")
            ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
            before = run.n_records
            consume(ring, run, collect, release, on_record)
            if ring.last_drain_status == B.OK:
                break
            if run.n_records == before and not release:
                break           # host ring full and the caller keeps the records
        run.stats = ring.get_stats()
    finally:
        if own:
            s.synchronize()
            ring.destroy()
    return run
