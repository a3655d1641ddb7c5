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


def _same_arr(x, y) -> bool:
    return (x is None and y is None) or (x is not None and y is not None and np.array_equal(x, y))


def batchable(a, b) -> bool:
    """Can call b ride in the same launch as call a?  Same layout, selection and transform."""
    if (a.paged is None) != (b.paged is None):
        return False
    ta, tb = a.tensor, b.tensor
    if ta.dtype != tb.dtype or tuple(ta.shape) != tuple(tb.shape) or tuple(ta.stride()) != tuple(tb.stride()):
        return False
    if a.out_dtype != b.out_dtype or a.summary_mask != b.summary_mask or a.step_id != b.step_id:
        return False
    if not (np.array_equal(a.reqs, b.reqs) and _same_arr(a.keep_mask, b.keep_mask)
            and _same_arr(a.row_index, b.row_index)):
        return False
    if a.paged is not None:
        pa, pb = a.paged, b.paged
        if (pa.block_size, pa.n_heads, pa.head_dim, list(pa.heads_sel)) != (pb.block_size, pb.n_heads, pb.head_dim,
                                                                            list(pb.heads_sel)):
            return False
        if pa.block_table is not pb.block_table and not torch.equal(pa.block_table, pb.block_table):
            return False
    return True


def group_calls(calls, max_batch: int):
    """Consecutive calls of a step that can share a launch, in hook order."""
    groups: List[list] = []
    for c in calls:
        if groups and len(groups[-1]) < max_batch and batchable(groups[-1][0], c):
            groups[-1].append(c)
        else:
            groups.append([c])
    return groups


def observe_group(ring: B.Ring, group, stream_handle: int, keep_alive: list, allow=()):
    """One dmi_observe_batch / dmi_observe_paged_batch for a group of calls -> (status, n_done)."""
    c = group[0]
    dev = c.tensor.device
    km = ri = None
    if c.keep_mask is not None:
        km = torch.from_numpy(np.ascontiguousarray(c.keep_mask, dtype=np.uint8)).to(dev)
        keep_alive.append(km)
    if c.row_index is not None:
        ri = torch.from_numpy(np.ascontiguousarray(c.row_index, dtype=np.int32)).to(dev)
        keep_alive.append(ri)
    return ring.observe_batch([g.point_id for g in group], [g.tensor for g in group], c.reqs, step_id=c.step_id,
                              stream=stream_handle, out_dtype=c.out_dtype, summary_mask=c.summary_mask,
                              keep_mask=km, row_index=ri, paged=c.paged, allow=allow)


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
                     bg_min_bytes: int = 0, before_observe: Optional[Callable] = None,
                     batch: int = 0, run: Optional[GpuRun] = None) -> GpuRun:
    """Lockstep schedule (the one the oracle's model follows): a step's observes,
    then every `drain_every` steps a flush-drain followed by poll + release.
    With lockstep=False the drain after a step moves only what has committed by
    then, without waiting for the step's kernels.  batch > 0: consecutive calls of
    a step that share layout, selection and transform go out together through
    dmi_observe_batch, at most `batch` per call.  run: a GpuRun to fill in (so that an
    on_record callback can look at run.launched while the workload is still running)."""
    own = ring is None
    if own:
        ring = B.Ring(device_ring_bytes or wl.device_ring_bytes, host_ring_bytes or wl.host_ring_bytes,
                      flags=flags, max_reqs_per_observe=wl.max_reqs, block_timeout_ms=block_timeout_ms,
                      bg_min_bytes=bg_min_bytes)
        ring.set_policy(wl.policy_mode, wl.sample_k, 0)
    if poison is not None:
        ring.debug_fill_rings(poison)
    run = GpuRun() if run is None else run
    s = torch.cuda.current_stream()
    keep_alive: list = []
    try:
        for step, calls in wl.steps():
            if max_steps is not None and step >= max_steps:
                break
            for group in (group_calls(calls, batch) if batch else ()):
                if before_observe is not None:
                    for c in group:
                        before_observe(c, s.cuda_stream)
                tries = 0
                while group:
                    rc, done = observe_group(ring, group, s.cuda_stream, keep_alive,
                                             allow=(B.ERR_AGAIN,) if tries < 200000 else ())
                    if rc == B.OK:
                        # disabled points are skipped inside the call; the oracle's driver lists what ran
                        run.launched.extend(c for c in group[:done])
                    group = group[done:]
                    if rc == B.ERR_AGAIN:
                        # completeness policy, no room: this thread is also the consumer
                        consume(ring, run, collect, release, on_record)
                        tries += 1
            for c in (() if batch else calls):
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


def run_workload_graph(wl, *, n_graph: Optional[int] = None, drain_every: int = 1, release: bool = True,
                       flags: int = 0, device_ring_bytes=None, host_ring_bytes=None, lockstep: bool = True,
                       block_timeout_ms: int = 1, bg_min_bytes: int = 0, replays_per_capture: int = 0,
                       batch: int = 0) -> GpuRun:
    """Feed a host-side workload whose steps repeat a fixed list of observes through
    a captured graph: the first `n_graph` calls of step 0 are captured once
    (torch.cuda.graph over dmi_step_observe launches on static device buffers); every
    step copies its tensor contents, keep vectors, row indices and block tables into
    those buffers, hands changed request tables to dmi_step_update, and replays the
    graph between dmi_step_begin and dmi_step_end.  Calls beyond the first n_graph of
    a step go through dmi_observe.  replays_per_capture > 0 re-captures the graph
    (a new step object) after that many replays.  batch > 0: consecutive fixed calls that
    share layout, selection and transform are captured as one dmi_step_observe_batch
    launch (at most `batch` of them); their keep vector, row indices and block table are
    then the first one's static buffers."""
    dev = "cuda:0"
    n_graph = wl.notes["n_graph"] if n_graph is None else n_graph
    ring = B.Ring(device_ring_bytes or wl.device_ring_bytes, host_ring_bytes or wl.host_ring_bytes,
                  flags=flags, max_reqs_per_observe=wl.max_reqs, block_timeout_ms=block_timeout_ms,
                  bg_min_bytes=bg_min_bytes)
    ring.set_policy(wl.policy_mode, wl.sample_k, 0)
    run = GpuRun()
    s = torch.cuda.current_stream()
    calls0 = wl.step_calls(0)[:n_graph]

    class Static:                       # device buffers of one fixed launch
        def __init__(self, c):
            self.tensor = c.tensor.to(dev)
            self.keep = None if c.keep_mask is None else torch.zeros(len(c.keep_mask), dtype=torch.uint8, device=dev)
            self.rows = None if c.row_index is None else torch.zeros(len(c.row_index), dtype=torch.int32, device=dev)
            self.table = None if c.paged is None else c.paged.block_table.to(dev)
            self.reqs = None

        def load(self, c):
            self.tensor.copy_(c.tensor)
            if self.keep is not None:
                self.keep.copy_(torch.from_numpy(np.ascontiguousarray(c.keep_mask, dtype=np.uint8)))
            if self.rows is not None:
                self.rows.copy_(torch.from_numpy(np.ascontiguousarray(c.row_index, dtype=np.int32)))
            if self.table is not None:
                self.table.copy_(c.paged.block_table)

    statics = [Static(c) for c in calls0]
    groups0 = group_calls(calls0, batch) if batch else [[c] for c in calls0]

    def capture():
        step = B.Step(ring, max(1, n_graph))
        graph = torch.cuda.CUDAGraph()
        step.capture_begin()
        with torch.cuda.graph(graph):
            h = torch.cuda.current_stream().cuda_stream
            pos = 0
            for grp in groups0:
                sts = statics[pos: pos + len(grp)]
                pos += len(grp)
                c, st = grp[0], sts[0]
                if len(grp) > 1:
                    spec = None
                    if c.paged is not None:
                        p = c.paged
                        spec = type(p)(p.block_size, p.n_heads, p.head_dim, p.heads_sel, st.table)
                    first = step.observe_batch([g.point_id for g in grp], [x.tensor for x in sts], c.reqs, stream=h,
                                               out_dtype=c.out_dtype, summary_mask=c.summary_mask, keep_mask=st.keep,
                                               row_index=st.rows, paged=spec)
                    for i, x in enumerate(sts):
                        x.node = first + i if first >= 0 else -1
                        x.reqs = np.array(c.reqs, copy=True)
                    continue
                if c.paged is None:
                    node = step.observe_tensor(c.point_id, st.tensor, c.reqs, stream=h, out_dtype=c.out_dtype,
                                               summary_mask=c.summary_mask, keep_mask=st.keep, row_index=st.rows)
                else:
                    p = c.paged
                    node = step.observe_paged(c.point_id, st.tensor, st.table, c.reqs, block_size=p.block_size,
                                              n_heads=p.n_heads, head_dim=p.head_dim, heads_sel=p.heads_sel,
                                              stream=h, out_dtype=c.out_dtype, summary_mask=c.summary_mask,
                                              keep_mask=st.keep)
                st.node = node
                st.reqs = np.array(c.reqs, copy=True)
        step.seal()
        return step, graph

    step, graph = capture()
    old = []
    replays = 0
    keep_alive: list = []
    try:
        for sidx, calls in wl.steps():
            if replays_per_capture and replays == replays_per_capture:
                old.append((step, graph))           # destroyed once its replays have finished
                step, graph = capture()
                replays = 0
            for c, st in zip(calls[:n_graph], statics):
                st.load(c)
                if st.node >= 0 and not np.array_equal(st.reqs, c.reqs):
                    step.update(st.node, c.reqs)
                    # launches captured with the same table follow it
                    for other in statics:
                        if other is not st and other.reqs is not None and np.array_equal(other.reqs, st.reqs):
                            other.reqs = np.array(c.reqs, copy=True)
                    st.reqs = np.array(c.reqs, copy=True)
            rc = step.begin(sidx, s.cuda_stream, allow=(B.ERR_AGAIN,))
            tries = 0
            while rc == B.ERR_AGAIN:
                consume(ring, run, True, release)
                tries += 1
                rc = step.begin(sidx, s.cuda_stream, allow=(B.ERR_AGAIN,) if tries < 200000 else ())
            graph.replay()
            step.end(s.cuda_stream)
            replays += 1
            if rc == B.OK:
                run.launched.extend(c for c, st in zip(calls[:n_graph], statics) if st.node >= 0)
            for c in calls[n_graph:]:
                c_dev = type(c)(**{**c.__dict__, "tensor": c.tensor.to(dev)})
                keep_alive.append(c_dev.tensor)
                rc = observe_call(ring, c_dev, s.cuda_stream, keep_alive, allow=(B.ERR_AGAIN,))
                tries = 0
                while rc == B.ERR_AGAIN:
                    consume(ring, run, True, release)
                    tries += 1
                    rc = observe_call(ring, c_dev, s.cuda_stream, keep_alive,
                                      allow=(B.ERR_AGAIN,) if tries < 200000 else ())
                if rc == B.OK:
                    run.launched.append(c)
            if (sidx + 1) % drain_every == 0:
                if lockstep:
                    s.synchronize()
                ring.drain(B.DRAIN_FLUSH if lockstep else 0, allow=(B.ERR_AGAIN,))
                consume(ring, run, True, release)
            else:
                s.synchronize()     # the next step overwrites the static buffers
        s.synchronize()
        deadline = time.monotonic() + 60.0
        while True:
            if time.monotonic() > deadline:
                raise RuntimeError("final drain made no progress for 60 s")
            ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
            before = run.n_records
            consume(ring, run, True, release)
            if ring.last_drain_status == B.OK:
                break
            if run.n_records == before and not release:
                break
        run.stats = ring.get_stats()
    finally:
        s.synchronize()
        for st_, g_ in old + [(step, graph)]:
            del g_
            st_.destroy()
        ring.destroy()
    return run
