#!/usr/bin/env python3
"""Benchmark of the capture-and-stage path on one MI355X.

Headline workload: the largest single-GPU configuration, "saturation" (config 5):
a Llama-70B-shaped decode step with 80 observation points (the residual stream of
every layer), 256 requests x 1 row x 8192 bf16 each, device ring 4 GiB, pinned host
ring 16 GiB, drop-newest, every step sampled (k = 1).  A step is one pass of the whole
hot path: the synthetic decode step (80 bf16 weight-streaming layers, one GPU's
tensor-parallel share), the policy gate, admission, slot reservation, gather + pack of
the step's 80 tensors (one batched launch at the end of the step), header and commit, the
drain into the pinned host ring (the library's drain thread, copy engine), host poll and
release.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

Also measured in the same run: the capture kernels of every workload shape, launched singly
and batched, against the HBM roofline (HIP events on the launch stream); the drain against
the box's own pinned D2H rate; step-time overhead against the no-capture step for configs
2, 3 and 5 (in line, batched, graph-replayed); the other configurations end to end; the
exporter stages; the front end's host cost per hook; and the CPU oracle on this machine's host
cores (a reported baseline, not the target).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X published HBM3E bandwidth
SEED_NOTE = "synthetic (seeded ~N(0,1) bf16, shapes of the paper's LLM workloads)"
# HBM bytes per launch of the batched config-5 capture kernel when it keeps all 80 records, from
# the two rocprofv3 --pmc runs summarised in profiles/hbm_traffic_counters.md (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size):
# 335.79 MB read + 339.63 MB written, against 671.83 MB algorithmic.
TRAFFIC_CONFIG5_BATCH80_BYTES = 675418753


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Ctx:
    """What every section needs: the libraries, the stream, small helpers."""

    def __init__(self):
        import numpy as np
        import torch
        import paper_2605_11093_amd as dmi
        from paper_2605_11093_amd import binding as B
        from workloads import configs
        self.np, self.torch, self.dmi, self.B, self.configs = np, torch, dmi, B, configs
        assert torch.cuda.is_available(), "bench.py needs the GPU"
        self.dev = "cuda:0"
        torch.cuda.set_device(0)
        dmi.lib()
        bench_so = os.path.join(ROOT, "paper_2605_11093_amd", "libdmi_bench.so")
        if not os.path.exists(bench_so):        # normally built beforehand by __graft_entry__.build()
            from paper_2605_11093_amd import build as _b
            _b.build_bench()
        bl = C.CDLL(bench_so)
        bl.dmi_bench_sleep.argtypes = [C.c_void_p, C.c_uint32]
        bl.dmi_bench_stream_gemv.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        bl.dmi_bench_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        self.bl = bl
        hip = C.CDLL("libamdhip64.so")
        hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        hip.hipEventSynchronize.argtypes = [C.c_void_p]
        hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.hip = hip
        self.stream = torch.cuda.current_stream()
        self.sh = self.stream.cuda_stream
        self.d2h_peak = None

    def ev_pair(self):
        t = self.torch
        return t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)

    def hw_ev_pair(self):
        """Two raw hipEvent_t handles for dmi_debug_time_next_launch (the kernel's own start and end)."""
        out = []
        for _ in range(2):
            e = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(e)) == 0
            out.append(e)
        return tuple(out)

    def hw_elapsed_us(self, k0, k1):
        assert self.hip.hipEventSynchronize(k1) == 0
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), k0, k1)
        assert rc == 0, f"hipEventElapsedTime: {rc}"
        return ms.value * 1e3

    def consume(self, ring):
        n = 0
        while True:
            k, views = ring.poll_host_raw()
            if not k:
                return n
            n += k
            ring.release_host(views[k - 1].seq)

    def settle(self, ring):
        B = self.B
        self.stream.synchronize()
        for _ in range(1000000):
            ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
            self.consume(ring)
            if ring.last_drain_status == B.OK:
                return
        raise RuntimeError("ring did not settle")

    def check(self, rc):
        rc = rc[0] if isinstance(rc, tuple) else rc
        if rc < 0:
            raise self.dmi.DmiError(rc, self.dmi.lib().dmi_last_error().decode())

    def free(self):
        self.torch.cuda.synchronize()
        self.torch.cuda.empty_cache()


# ---------------------------------------------------------------------- kernel timing
def time_launches(ctx, make_call, n_launch, ring_bytes, alg_bytes, reps=3, max_reqs=256, policy=None):
    """n_launch captures queued behind a sleeping stream so that they run back to back; HIP
    events on the same stream bracket them.  The ring holds every launch, so the completeness
    policy never waits and its commit probes are events only.  Returns the mean over `reps`
    repetitions (and the best) of microseconds per launch, and (us_kernel) the mean duration of the
    kernels themselves in one more repetition, first launch left out."""
    B = ctx.B
    per = []
    for rep in range(reps + 1):
        ring = B.Ring(ring_bytes, max(1 << 26, (alg_bytes + 63) // 64 * 64), max_reqs_per_observe=max_reqs)
        ring.set_policy(B.POLICY_BLOCK if policy is None else policy)
        po = make_call(ring)
        if rep == 0:                                    # warm-up: code objects, allocator
            for i in range(2):
                ctx.check(po(i, ctx.sh))
            ctx.stream.synchronize()
            ring.destroy()
            continue
        e0, e1 = ctx.ev_pair()
        ctx.bl.dmi_bench_sleep(ctx.sh, 300 + 20 * n_launch)
        e0.record(ctx.stream)
        for i in range(n_launch):
            ctx.check(po(i, ctx.sh))
        e1.record(ctx.stream)
        e1.synchronize()
        per.append(e0.elapsed_time(e1) * 1e3 / n_launch)
        st = ring.get_stats()
        assert st.dropped_records == 0, st
        ring.destroy()
    mean = sum(per) / len(per)
    # once more with every launch timed by the hardware itself (its own start and end stamps):
    # the kernel's duration without the gap to the next dispatch
    ring = B.Ring(ring_bytes, max(1 << 26, (alg_bytes + 63) // 64 * 64), max_reqs_per_observe=max_reqs)
    ring.set_policy(B.POLICY_BLOCK if policy is None else policy)
    po = make_call(ring)
    pairs = [ctx.hw_ev_pair() for _ in range(n_launch)]
    ctx.bl.dmi_bench_sleep(ctx.sh, 300 + 20 * n_launch)
    for i in range(n_launch):
        B.time_next_launch(*pairs[i])
        ctx.check(po(i, ctx.sh))
    ctx.stream.synchronize()
    own = [ctx.hw_elapsed_us(k0, k1) for k0, k1 in pairs]
    for k0, k1 in pairs:
        ctx.hip.hipEventDestroy(k0)
        ctx.hip.hipEventDestroy(k1)
    ring.destroy()
    kern = sum(own[1:]) / len(own[1:]) if len(own) > 1 else own[0]
    return {"us_per_launch": round(mean, 3), "us_per_launch_best": round(min(per), 3),
            "algorithmic_bytes": alg_bytes, "GBs": round(alg_bytes / mean / 1e3, 1),
            "frac_hbm_peak": round(alg_bytes / mean / 1e3 / HBM_PEAK_GBS, 4),
            "us_kernel": round(kern, 3), "frac_hbm_peak_kernel": round(alg_bytes / kern / 1e3 / HBM_PEAK_GBS, 4)}


def shape_table(ctx):
    """Every workload shape's capture launch: name -> (make_call(ring), algorithmic bytes,
    launches per timing, ring bytes, cleanup).  Built lazily, one shape at a time, because the
    inputs of the larger ones take tens of GiB."""
    dmi, B, configs, np, torch, dev = ctx.dmi, ctx.B, ctx.configs, ctx.np, ctx.torch, ctx.dev

    def c1():
        w = configs.config1_tiny(device=dev, n_steps=1)
        calls = w.step_calls(0)
        c = calls[0]
        alg = 4 * 256 * 4 + 4 * 36 + 64
        yield "config1_record", lambda r: dmi.PreparedObserve(r, c.point_id, c.tensor, c.reqs), alg, 256, 2176 * 260 + (1 << 20)
        yield ("config1_batch8", lambda r: dmi.PreparedBatch(r, [x.point_id for x in calls], [x.tensor for x in calls], c.reqs),
               alg * 8, 64, 2176 * 8 * 66 + (1 << 20))

    def c2():
        w = configs.config2_decode8b(device=dev, n_steps=1)
        calls = w.step_calls(0)
        c = calls[0]
        rb = dmi.record_bytes(64, 64, 4096, B.DT_BF16, 5)
        alg = rb + 64 * 4096 * 2 + 64 * 20
        yield ("config2_record", lambda r: dmi.PreparedObserve(r, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype,
                                                                 summary_mask=c.summary_mask), alg, 256, rb * 260 + (1 << 20))
        km = torch.from_numpy((np.arange(64) % 4 != 1).astype(np.uint8)).to(dev)
        kept = int((np.arange(64) % 4 != 1).sum())
        yield ("config2_record_keep_vector",
               lambda r: dmi.PreparedObserve(r, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype,
                                             summary_mask=c.summary_mask, keep_mask=km),
               kept * 4096 * 4 + 64 * 37 + 64 + kept * 8, 256, rb * 260 + (1 << 20))
        yield ("config2_batch32", lambda r: dmi.PreparedBatch(r, [x.point_id for x in calls], [x.tensor for x in calls],
                                                                 c.reqs, out_dtype=c.out_dtype, summary_mask=c.summary_mask),
               alg * 32, 16, rb * 32 * 18 + (1 << 20))

    def c3():
        w = configs.config3_prefill(device=dev, n_steps=1)
        calls = w.step_calls(0)
        res = [x for x in calls if x.point_id < 100]
        mlp = [x for x in calls if x.point_id >= 100]
        rows = int(res[0].reqs[:, 3].sum())
        for nm, grp, E in (("resid", res, 4096), ("mlp", mlp, 14336)):
            alg = rows * E * 3 + 32 * 36 + 64
            rb = dmi.record_bytes(32, rows, E, B.DT_FP8, 0)
            g0 = grp[0]
            yield (f"config3_{nm}_fp8", lambda r, g0=g0: dmi.PreparedObserve(r, g0.point_id, g0.tensor, g0.reqs, out_dtype=B.DT_FP8),
                   alg, 8, rb * 10)
            if nm == "resid":
                # the same rows' worth of bytes from consecutive tokens instead of every fourth: does the
                # stride through the source cost anything?
                dense = g0.reqs.copy()
                dense[:, 4] = 1
                yield ("config3_resid_fp8_consecutive_tokens",
                       lambda r, g0=g0, dense=dense: dmi.PreparedObserve(r, g0.point_id, g0.tensor, dense, out_dtype=B.DT_FP8),
                       alg, 8, rb * 10)
            yield (f"config3_{nm}_fp8_batch{len(grp)}",
                   lambda r, grp=grp, g0=g0: dmi.PreparedBatch(r, [x.point_id for x in grp], [x.tensor for x in grp], g0.reqs,
                                                               out_dtype=B.DT_FP8), alg * len(grp), 4, rb * len(grp) * 6)

    def c4():
        w = configs.config4_paged_kv(device=dev, n_steps=1)
        calls = w.step_calls(0)
        c = calls[0]
        rows = int(c.reqs[:, 3].sum())
        alg = rows * 256 * 4 + rows // 16 * 4 + 16 * 36 + 64
        rb = dmi.record_bytes(16, rows, 256, B.DT_BF16, 0)
        yield ("config4_kv_slice", lambda r: dmi.PreparedObserve(r, c.point_id, c.tensor, c.reqs, paged=c.paged), alg, 8, rb * 10)
        yield ("config4_kv_batch8", lambda r: dmi.PreparedBatch(r, [x.point_id for x in calls], [x.tensor for x in calls], c.reqs,
                                                                   paged=c.paged), alg * 8, 6, rb * 8 * 8)

    def c5():
        w = configs.config5_saturation(device=dev, n_steps=1)
        calls = w.step_calls(0)
        c = calls[0]
        alg = 256 * 8192 * 4 + 256 * 36 + 64
        rb = dmi.record_bytes(256, 256, 8192, B.DT_BF16, 0)
        yield "config5_record", lambda r: dmi.PreparedObserve(r, c.point_id, c.tensor, c.reqs), alg, 64, rb * 68
        for nb in (8, 80):
            cs = calls[:nb]
            yield (f"config5_batch{nb}", lambda r, cs=cs: dmi.PreparedBatch(r, [x.point_id for x in cs], [x.tensor for x in cs], c.reqs),
                   alg * nb, 8, rb * nb * 10)
        # the same launch under the best-effort policy (nothing dropped: the ring holds every launch)
        yield (f"config5_batch80_drop_newest", lambda r: dmi.PreparedBatch(r, [x.point_id for x in calls], [x.tensor for x in calls], c.reqs),
               alg * 80, 8, rb * 80 * 10, B.POLICY_DROP_NEWEST)

    return {"config1": c1, "config2": c2, "config3": c3, "config4": c4, "config5": c5}


def run_kernel_table(ctx, only=None, profile=False):
    """Times every shape (or, for a profiler run, launches one shape a fixed number of times)."""
    out = {}
    for cfg, gen in shape_table(ctx).items():
        if only is not None and not any(o.startswith(cfg) for o in only):
            continue
        for name, make, alg, n_launch, ring_bytes, *rest in gen():
            policy = rest[0] if rest else ctx.B.POLICY_BLOCK
            if only is not None and name not in only:
                continue
            if profile:
                ring = ctx.B.Ring(ring_bytes, max(1 << 26, (alg + 63) // 64 * 64), max_reqs_per_observe=256)
                ring.set_policy(policy)
                po = make(ring)
                for i in range(n_launch):
                    ctx.check(po(i, ctx.sh))
                ctx.stream.synchronize()
                ring.destroy()
                log(f"profiled shape {name}: {n_launch} launches of {alg} algorithmic bytes each")
            else:
                out[name] = time_launches(ctx, make, n_launch, ring_bytes, alg, policy=policy)
                log(f"kernel {name}: {out[name]}")
        ctx.free()
    return out


# ---------------------------------------------------------------------- probes
def run_probes(ctx, extra):
    torch, dev, stream = ctx.torch, ctx.dev, ctx.stream
    a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    hp = torch.empty(1 << 30, dtype=torch.uint8, pin_memory=True)
    best = 1e9
    for _ in range(5):
        e0, e1 = ctx.ev_pair()
        e0.record(stream)
        b.copy_(a)
        e1.record(stream)
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1))
    d2d = 2 * (1 << 30) / best / 1e6
    best = 1e9
    for _ in range(10):
        torch.cuda.synchronize()
        t = time.perf_counter()
        hp.copy_(a, non_blocking=True)
        torch.cuda.synchronize()
        best = min(best, time.perf_counter() - t)
    ctx.d2h_peak = (1 << 30) / best / 1e9
    del a, b, hp
    ctx.free()
    log(f"probes: device copy {d2d:.0f} GB/s (read+write), pinned D2H {ctx.d2h_peak:.1f} GB/s")
    extra["hbm_copy_probe_GBs"] = round(d2d, 1)
    extra["pinned_d2h_peak_GBs"] = round(ctx.d2h_peak, 2)


def run_second_queue_probe(ctx, extra):
    """What a waiting launch on a second hardware queue costs the producer's dispatches (the
    reason why nothing of the library runs on a second compute queue while captures are in
    flight): 256 plain 512 KiB copy kernels back to back, alone, and while a launch on
    another stream waits for an event of this one."""
    torch, dev, stream, sh, bl = ctx.torch, ctx.dev, ctx.stream, ctx.sh, ctx.bl
    src_q = torch.empty(512 << 10, dtype=torch.uint8, device=dev)
    dst_q = torch.empty(512 << 10, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    q = {}
    for name, busy in (("alone", False), ("second_queue_waiting", True)):
        best = 1e9
        for rep in range(4):
            torch.cuda.synchronize()
            e0, e1 = ctx.ev_pair()
            bl.dmi_bench_sleep(sh, 3000)
            e0.record(stream)
            for i in range(256):
                bl.dmi_bench_copy(dst_q.data_ptr(), src_q.data_ptr(), 512 << 10, sh)
            e1.record(stream)
            if busy:
                side.wait_event(e1)
                bl.dmi_bench_sleep(side.cuda_stream, 1)
            e1.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / 256)
            torch.cuda.synchronize()
        q[name] = round(best, 3)
    extra["dispatch_us_per_512KiB_copy_kernel"] = q
    log(f"512 KiB copy kernels back to back: {q} us per launch")


# ---------------------------------------------------------------------- config 5 (headline)
class Config5:
    """The saturation workload with its interfering decode step: 80 layers of a 70B model's
    TP-8 share (219 MB of bf16 weights each) stream through a GEMV; 320 MiB per captured
    step exceed what the host link takes in the step's time."""
    N_L, N_W = 80, 219 * 1000 * 1000 // 2 // 8 * 8
    ALG_PER_RECORD = 256 * 8192 * 4 + 256 * 36 + 64

    def __init__(self, ctx):
        torch, dev = ctx.torch, ctx.dev
        self.ctx = ctx
        self.w = ctx.configs.config5_saturation(device=dev, n_steps=4)
        self.calls = [self.w.step_calls(s) for s in range(4)]           # the pool has 4 slots per point
        self.weights = [torch.empty(self.N_W, dtype=torch.bfloat16, device=dev).normal_() for _ in range(self.N_L)]
        self.xv = torch.randn(4096, device=dev).to(torch.bfloat16)
        self.ac = torch.zeros(4096, dtype=torch.float32, device=dev)
        self.ring = ctx.B.Ring(self.w.device_ring_bytes, self.w.host_ring_bytes, flags=ctx.B.BG_THREAD,
                               max_reqs_per_observe=256)
        dmi = ctx.dmi
        self.single = [[dmi.PreparedObserve(self.ring, c.point_id, c.tensor, c.reqs) for c in self.calls[s]]
                       for s in range(4)]
        self.batched = [dmi.PreparedBatch(self.ring, [c.point_id for c in self.calls[s]],
                                          [c.tensor for c in self.calls[s]], self.calls[s][0].reqs) for s in range(4)]
        self.rec_bytes = dmi.record_bytes(256, 256, 8192, ctx.B.DT_BF16, 0)
        self.base_s = None
        # a decode loop cannot run far ahead of its own sampled tokens: at most DEPTH steps are in flight
        self.DEPTH = 2
        self.step_done = [torch.cuda.Event() for _ in range(self.DEPTH)]
        self.n_issued = 0

    def layer(self, l):
        self.ctx.bl.dmi_bench_stream_gemv(self.weights[l].data_ptr(), self.N_W, self.xv.data_ptr(),
                                          self.ac.data_ptr(), self.ctx.sh)

    def steps(self, first, count, mode, events=None):
        """mode: None (no capture), 'inline' (an observe behind every layer), 'batched' (one
        dmi_observe_batch for the step's 80 tensors once the last layer has run)."""
        ctx = self.ctx
        for s in range(first, first + count):
            slot = self.n_issued % self.DEPTH
            if self.n_issued >= self.DEPTH:
                self.step_done[slot].synchronize()      # step n - DEPTH has finished
            self.n_issued += 1
            for l in range(self.N_L):
                self.layer(l)
                if mode == "inline":
                    ctx.check(self.single[s % 4][l](s, ctx.sh))
            if mode == "batched":
                ev = events[s - first] if events is not None else None
                if ev is not None:
                    e0, e1, k0, k1 = ev
                    e0.record(ctx.stream)
                    ctx.B.time_next_launch(k0, k1)      # the launch's own start and end, by the hardware
                ctx.check(self.batched[s % 4](s, ctx.sh))
                if ev is not None:
                    e1.record(ctx.stream)
            elif mode is None and events is not None and events[s - first] is not None:
                e0, e1 = events[s - first][:2]          # what the bracket itself measures, with nothing in it
                e0.record(ctx.stream)
                e1.record(ctx.stream)
            self.step_done[slot].record(ctx.stream)
            if mode:
                ctx.consume(self.ring)

    def baseline(self):
        torch = self.ctx.torch
        self.steps(0, 3, None)
        torch.cuda.synchronize()
        t = time.perf_counter()
        self.steps(0, 20, None)
        torch.cuda.synchronize()
        self.base_s = (time.perf_counter() - t) / 20
        evs = [self.ctx.ev_pair() for _ in range(20)]
        self.steps(0, 20, None, evs)
        torch.cuda.synchronize()
        self.empty_bracket_us = sum(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs) / len(evs)
        return self.base_s

    def run(self, k, mode, n_steps, warmup=0, events=False, first_step=0):
        """n_steps steps (step ids from first_step on) at 1-in-k sampling.  Timed from a
        synchronised start until everything captured has been delivered to the consumer."""
        ctx, B, ring = self.ctx, self.ctx.B, self.ring
        ring.set_policy(B.POLICY_DROP_NEWEST, k, 0)
        if warmup:
            self.steps(first_step, warmup, mode)
        ctx.settle(ring)
        a0 = ring.get_stats()
        # every launch of the region is timed: a sample of them would need each launch's own byte count,
        # and how many records a launch keeps varies from step to step (timing a launch costs the
        # stream some 10 us, 0.3 % of a step, which the region's step time and overhead include)
        evs = [ctx.ev_pair() + ctx.hw_ev_pair() for i in range(n_steps)] if events else None
        ctx.torch.cuda.synchronize()
        t = time.perf_counter()
        self.steps(first_step + warmup, n_steps, mode, evs)
        ctx.stream.synchronize()
        t_stream = time.perf_counter() - t
        a1 = ring.get_stats()
        ctx.settle(ring)
        ctx.torch.cuda.synchronize()
        t_all = time.perf_counter() - t
        a2 = ring.get_stats()
        cap, drp = a2.captured_bytes - a0.captured_bytes, a2.dropped_bytes - a0.dropped_bytes
        res = {"delivered_GBs": round((a2.released_bytes - a0.released_bytes) / t_all / 1e9, 3),
               "drained_GBs_while_stepping": round((a1.drained_bytes - a0.drained_bytes) / t_stream / 1e9, 2),
               "dropped_fraction": round(drp / (cap + drp), 4) if cap + drp else 0.0,
               "ms_per_step": round(t_all / n_steps * 1e3, 4),
               "ms_per_step_stream": round(t_stream / n_steps * 1e3, 4),
               "captured_records": a2.captured_records - a0.captured_records,
               "dropped_records": a2.dropped_records - a0.dropped_records,
               "released_bytes": a2.released_bytes - a0.released_bytes}
        if self.base_s:
            res["overhead_pct"] = round((t_stream / n_steps - self.base_s) / self.base_s * 100, 2)
        if evs:
            evs = [e for e in evs if e is not None]
            us = [e0.elapsed_time(e1) * 1e3 for e0, e1, _, _ in evs]
            hw = [ctx.hw_elapsed_us(k0, k1) for _, _, k0, k1 in evs]
            res["launch_us_mean"] = sum(hw) / len(hw)
            res["launch_us_min"] = min(hw)
            res["launch_us_max"] = max(hw)
            res["launch_us_between_events_mean"] = sum(us) / len(us)
            res["launches"] = n_steps
            res["launches_timed"] = len(us)
        return res

    def request_granular(self, n_steps):
        """The same overload met request by request (the paper's best-effort policy, drop-recent):
        before every step a policy manager on the host sizes a keep vector to what the host link
        takes in one step (95 % of the measured pinned D2H rate over the step time; halved while
        the ring's guaranteed room is under a quarter), most recently admitted requests out first;
        the capture kernels gather only the kept requests.  Whole records should no longer drop."""
        ctx, B, dmi, np, ring = self.ctx, self.ctx.B, self.ctx.dmi, self.ctx.np, self.ring
        ring.set_policy(B.POLICY_DROP_NEWEST, 1, 0)
        ctx.settle(ring)
        n_r = self.calls[0][0].reqs.shape[0]

        class _Ptr:                     # a device address where the binding expects a tensor
            def __init__(self, p):
                self.p = p

            def data_ptr(self):
                return self.p

        ones = np.ones(n_r, dtype=np.uint8)
        by_mask = {}
        for _ in range(4):              # the library rotates over four keep-vector buffers
            ptr = ring.set_keep_mask(ones, ctx.sh)
            by_mask[ptr] = [dmi.PreparedBatch(ring, [c.point_id for c in self.calls[s]], [c.tensor for c in self.calls[s]],
                                              self.calls[s][0].reqs, keep_mask=_Ptr(ptr)) for s in range(4)]
        req_info = [(int(q[0]), 1, i, 0) for i, q in enumerate(self.calls[0][0].reqs)]
        a0 = ring.get_stats()
        kept_sum = 0
        ctx.torch.cuda.synchronize()
        t = time.perf_counter()
        for s in range(n_steps):
            budget = int(0.95 * ctx.d2h_peak * 1e9 * self.base_s * 1.08) // self.N_L
            if ring.free_bytes() < self.w.device_ring_bytes // 4:
                budget //= 2
            keep = B.policy_select(B.SELECT_DROP_RECENT, req_info, 8192 * 2, max(0, budget - 4160))
            kept_sum += int(keep.sum())
            po = by_mask[ring.set_keep_mask(keep, ctx.sh)][s % 4]
            slot = self.n_issued % self.DEPTH
            if self.n_issued >= self.DEPTH:
                self.step_done[slot].synchronize()
            self.n_issued += 1
            for l in range(self.N_L):
                self.layer(l)
            ctx.check(po(5000 + s, ctx.sh))
            self.step_done[slot].record(ctx.stream)
            ctx.consume(ring)
        ctx.stream.synchronize()
        dt = time.perf_counter() - t
        a1 = ring.get_stats()
        ctx.settle(ring)
        a2 = ring.get_stats()
        return {"drained_GBs": round((a1.drained_bytes - a0.drained_bytes) / dt / 1e9, 2),
                "requests_kept_fraction": round(kept_sum / (n_steps * n_r), 4),
                "whole_records_dropped": a2.dropped_records - a0.dropped_records,
                "ms_per_step": round(dt / n_steps * 1e3, 3),
                "overhead_pct": round((dt / n_steps - self.base_s) / self.base_s * 100, 2)}

    def close(self):
        self.ctx.stream.synchronize()
        self.ring.destroy()
        del self.weights, self.single, self.batched, self.calls, self.w
        self.ctx.free()


# ---------------------------------------------------------------------- config 2
def run_config2(ctx, extra, skip_overhead):
    """Llama-3-8B-shaped decode (config 2): whole path in line and batched, the drain engines,
    step-time overhead against 32 x 436 MB weight-streaming layers (in line, batched at step
    end, and with every step replayed from a graph), the exporter stages."""
    dmi, B, configs, torch, dev, stream, sh, bl = ctx.dmi, ctx.B, ctx.configs, ctx.torch, ctx.dev, ctx.stream, ctx.sh, ctx.bl
    n_points, n_reqs, hidden = 32, 64, 4096
    wl = configs.config2_decode8b(device=dev, n_steps=4)
    rec_bytes = dmi.record_bytes(n_reqs, n_reqs, hidden, B.DT_BF16, 5)
    step_bytes = rec_bytes * n_points
    calls0 = [wl.step_calls(s) for s in range(4)]

    def prepared(ring):
        return [[dmi.PreparedObserve(ring, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype,
                                     summary_mask=c.summary_mask) for c in calls0[slot]] for slot in range(4)]

    def prepared_batch(ring):
        return [dmi.PreparedBatch(ring, [c.point_id for c in calls0[slot]], [c.tensor for c in calls0[slot]],
                                  calls0[slot][0].reqs, out_dtype=calls0[slot][0].out_dtype,
                                  summary_mask=calls0[slot][0].summary_mask) for slot in range(4)]

    out = {"bytes_per_step": step_bytes}
    # -- whole path, no model in between: 32 observes (or one batch), drain thread, poll + release
    for mode in ("inline", "batched"):
        ring = B.Ring(wl.device_ring_bytes, wl.host_ring_bytes, flags=B.BG_THREAD, max_reqs_per_observe=256,
                      block_timeout_ms=2000)
        ring.set_policy(B.POLICY_BLOCK)
        pos, pob = prepared(ring), prepared_batch(ring)

        def run_steps(first, count):
            for s in range(first, first + count):
                if mode == "inline":
                    for po in pos[s % 4]:
                        ctx.check(po(s, sh))
                else:
                    ctx.check(pob[s % 4](s, sh))
                ctx.consume(ring)

        run_steps(0, 16)
        ctx.settle(ring)
        st0 = ring.get_stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(16, 256)
        ctx.settle(ring)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st1 = ring.get_stats()
        moved = st1.released_bytes - st0.released_bytes
        assert moved == step_bytes * 256 and st1.dropped_records == 0, (moved, st1)
        out[f"whole_path_{mode}"] = {"GBs": round(moved / dt / 1e9, 2), "ms_per_step": round(dt / 256 * 1e3, 4),
                                     "frac_of_d2h_peak": round(moved / dt / 1e9 / ctx.d2h_peak, 3)}
        log(f"config 2 whole path ({mode}): {out[f'whole_path_{mode}']}")
        ring.destroy()

    # -- drain alone, both engines
    drain = {}
    for name, fl in (("copy_engine", B.DRAIN_COPY_ENGINE), ("kernel", B.DRAIN_KERNEL)):
        r2 = B.Ring(wl.device_ring_bytes, wl.host_ring_bytes, flags=fl, max_reqs_per_observe=256)
        p2 = [po for slot in prepared(r2) for po in slot]
        rates = []
        for rep in range(4):
            for i in range(384):                                  # 202 MB committed, nothing drained
                ctx.check(p2[i % len(p2)](i, sh))
            stream.synchronize()
            t = time.perf_counter()
            n = r2.drain(B.DRAIN_FLUSH)
            dt = time.perf_counter() - t
            rates.append(n / dt / 1e9)
            while r2.poll_host():
                pass
            r2.release_host(r2.get_stats().launched_records)
        drain[name] = round(max(rates[1:]), 2)
        r2.destroy()
    log(f"drain alone: {drain} GB/s")
    extra["drain_GBs"] = drain
    extra["drain_frac_of_d2h_peak"] = {k: round(v / ctx.d2h_peak, 3) for k, v in drain.items()}

    if not skip_overhead:
        n_w = 436 * 1000 * 1000 // 2 // 8 * 8                  # one Llama-3-8B layer of bf16 weights
        weights = [torch.empty(n_w, dtype=torch.bfloat16, device=dev).normal_() for _ in range(n_points)]
        xvec = torch.randn(4096, device=dev).to(torch.bfloat16)
        acc = torch.zeros(4096, dtype=torch.float32, device=dev)
        r4 = B.Ring(wl.device_ring_bytes, wl.host_ring_bytes, flags=B.BG_THREAD, max_reqs_per_observe=256)
        p4, p4b = prepared(r4), prepared_batch(r4)

        def model_steps(first, count, capture):
            for s in range(first, first + count):
                for l in range(n_points):
                    bl.dmi_bench_stream_gemv(weights[l].data_ptr(), n_w, xvec.data_ptr(), acc.data_ptr(), sh)
                    if capture == "inline":
                        ctx.check(p4[s % 4][l](s, sh))
                if capture == "batched":
                    ctx.check(p4b[s % 4](s, sh))
                if capture:
                    ctx.consume(r4)

        per_step = {None: [], "inline": [], "batched": []}
        model_steps(0, 5, "inline")
        model_steps(0, 5, "batched")
        stream.synchronize()
        for rep in range(5):
            for capture in (None, "inline", "batched"):
                torch.cuda.synchronize()
                t = time.perf_counter()
                model_steps(100 + rep * 20, 20, capture)
                stream.synchronize()
                if capture:      # "including the tail of the offload path"
                    while r4.get_stats().drained_bytes < r4.get_stats().captured_bytes:
                        time.sleep(0.00005)
                    ctx.consume(r4)
                per_step[capture].append((time.perf_counter() - t) * 1e3 / 20)
        base = statistics.median(per_step[None])
        st = r4.get_stats()
        r4.destroy()
        ov = {"no_capture_ms_per_step": round(base, 4),
              "interfering_workload": "32 x 436 MB bf16 weight-streaming GEMV per step",
              "filler_GBs": round(n_points * n_w * 2 / base / 1e6, 1), "dropped_records": st.dropped_records,
              "paper_context": "0.4-6.8 % offline, ~6 % online on H100 (other hardware, real models)"}
        for capture in ("inline", "batched"):
            m = statistics.median(per_step[capture])
            ov[capture] = {"capture_ms_per_step": round(m, 4), "overhead_pct": round((m - base) / base * 100, 3),
                           "captured_GBs_during": round(step_bytes / m / 1e6, 2)}
        out["overhead"] = ov
        log(f"config 2 overhead: {ov}")

        # each step captured once into a graph and replayed (how a serving engine runs decode):
        # 32 x (GEMV + capture launch) per graph, or 32 GEMV + one batched capture launch
        r7 = B.Ring(wl.device_ring_bytes, wl.host_ring_bytes, flags=B.BG_THREAD, max_reqs_per_observe=256)

        def capture_graph(slot, with_gemv, mode_, ring_):
            step = B.Step(ring_, n_points) if mode_ else None
            g = torch.cuda.CUDAGraph()
            if step is not None:
                step.capture_begin()
            with torch.cuda.graph(g):
                h = torch.cuda.current_stream().cuda_stream
                for l in range(n_points):
                    if with_gemv:
                        bl.dmi_bench_stream_gemv(weights[l].data_ptr(), n_w, xvec.data_ptr(), acc.data_ptr(), h)
                    if mode_ == "inline":
                        c = calls0[slot][l]
                        step.observe_tensor(c.point_id, c.tensor, c.reqs, stream=h, out_dtype=c.out_dtype,
                                            summary_mask=c.summary_mask)
                if mode_ == "batched":
                    cs = calls0[slot]
                    step.observe_batch([c.point_id for c in cs], [c.tensor for c in cs], cs[0].reqs, stream=h,
                                       out_dtype=cs[0].out_dtype, summary_mask=cs[0].summary_mask)
            if step is not None:
                step.seal()
            return step, g

        g_base = capture_graph(0, True, None, None)[1]
        graphs = {m: [capture_graph(slot, True, m, r7) for slot in range(4)] for m in ("inline", "batched")}

        def graph_steps(first, count, capture):
            for s in range(first, first + count):
                if capture:
                    step, g = graphs[capture][s % 4]
                    step.begin(s, sh)
                    g.replay()
                    step.end(sh)
                    ctx.consume(r7)
                else:
                    g_base.replay()

        per_step = {None: [], "inline": [], "batched": []}
        for m in (None, "inline", "batched"):
            graph_steps(0, 5, m)
        stream.synchronize()
        for rep in range(5):
            for capture in (None, "inline", "batched"):
                torch.cuda.synchronize()
                t = time.perf_counter()
                graph_steps(100 + rep * 20, 20, capture)
                stream.synchronize()
                if capture:
                    while r7.get_stats().drained_bytes < r7.get_stats().captured_bytes:
                        time.sleep(0.00005)
                    ctx.consume(r7)
                per_step[capture].append((time.perf_counter() - t) * 1e3 / 20)
        base_g = statistics.median(per_step[None])
        st = r7.get_stats()
        assert st.dropped_records == 0 and st.captured_records == st.launched_records
        og = {"no_capture_ms_per_step": round(base_g, 4),
              "what": "each step one graph replay between dmi_step_begin and dmi_step_end: 32 x (GEMV + capture "
                      "launch), or 32 GEMV and one batched capture launch"}
        for capture in ("inline", "batched"):
            m = statistics.median(per_step[capture])
            og[capture] = {"capture_ms_per_step": round(m, 4), "overhead_pct": round((m - base_g) / base_g * 100, 3)}
        out["overhead_graph_replay"] = og
        log(f"config 2 overhead, graph replay: {og}")
        torch.cuda.synchronize()
        for lst in graphs.values():
            for step, g in lst:
                del g
                step.destroy()
        del graphs, g_base
        r7.destroy()
        del weights
        ctx.free()

    # -- exporter stages 2-3
    r6 = B.Ring(wl.device_ring_bytes, wl.host_ring_bytes, flags=B.BG_THREAD, max_reqs_per_observe=256)
    p6 = prepared_batch(r6)
    r6.exporter_start(1 << 30, 8)
    buf = (B.SliceC * 4096)()
    n_exp_steps, got_slices = 64, 0
    want_slices = n_exp_steps * n_points * n_reqs
    torch.cuda.synchronize()
    t = time.perf_counter()
    s6 = 0
    while got_slices < want_slices:
        if s6 < n_exp_steps:
            ctx.check(p6[s6 % 4](s6, sh))
            s6 += 1
        k = r6.exporter_next_many(buf, 1 if s6 < n_exp_steps else 1000)
        got_slices += k
        if k:
            r6.exporter_release_many(buf, k)
    dt = time.perf_counter() - t
    r6.exporter_stop()
    stream.synchronize()
    r6.destroy()
    extra["exporter"] = {"GBs": round(n_exp_steps * step_bytes / dt / 1e9, 2), "slices_per_s": round(got_slices / dt),
                         "what": "config 2 stream through capture, drain thread, pageable copy (8 workers), "
                                 "slice by request; Python consumer releasing in batches"}
    log(f"exporter: {extra['exporter']}")
    extra["config2_decode8b"] = out
    del wl, calls0
    ctx.free()


# ---------------------------------------------------------------------- configs 3 and 4 end to end
def run_configs34(ctx, extra):
    dmi, B, configs, torch, dev, stream, sh, bl = ctx.dmi, ctx.B, ctx.configs, ctx.torch, ctx.dev, ctx.stream, ctx.sh, ctx.bl
    from paper_2605_11093_amd.replay import run_workload_gpu
    e2e = {}

    def model_compute(call, stream_handle):
        # stand-in for the layers between two observation points: 2 ms of stream time
        bl.dmi_bench_sleep(stream_handle, 2000)

    def timed_replay(name, w, block_timeout_ms=2000, compute=True, batch=0):
        rr = B.Ring(w.device_ring_bytes, w.host_ring_bytes, flags=B.BG_THREAD,
                    max_reqs_per_observe=w.max_reqs, block_timeout_ms=block_timeout_ms)
        rr.set_policy(w.policy_mode, w.sample_k, 0)
        torch.cuda.synchronize()
        t = time.perf_counter()
        run = run_workload_gpu(w, collect=False, lockstep=False, ring=rr,
                               before_observe=model_compute if compute else None, batch=batch)
        dt = time.perf_counter() - t
        stt = run.stats
        rr.destroy()
        tot = stt.captured_bytes + stt.dropped_bytes
        base = None
        if compute:     # the same stand-in alone: one 2 ms sleep per observe
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(stt.observed_calls):
                bl.dmi_bench_sleep(sh, 2000)
            stream.synchronize()
            base = time.perf_counter() - t
        e2e[name] = {"drained_GBs": round(stt.drained_bytes / dt / 1e9, 2),
                     "frac_of_d2h_peak": round(stt.drained_bytes / dt / 1e9 / ctx.d2h_peak, 3),
                     "dropped_fraction": round(stt.dropped_bytes / tot, 4) if tot else 0.0,
                     "records": stt.launched_records, "seconds": round(dt, 3),
                     "model_compute_stand_in": "2 ms sleep kernel before every observe" if compute
                     else "none: captures issued back to back, the host link is the limit"}
        if base:
            e2e[name]["no_capture_seconds"] = round(base, 3)
            e2e[name]["overhead_pct"] = round((dt - base) / base * 100, 2)
        log(f"end to end {name}: {e2e[name]}")

    w3e = configs.config3_prefill(device=dev, n_steps=4)
    timed_replay("config3_prefill_4steps", w3e)
    timed_replay("config3_prefill_4steps_back_to_back", w3e, compute=False)
    # config 3 against a GEMM-bound prefill stand-in: one bf16 [tokens, 4096] x [4096, 4096] matmul
    # (torch / hipBLASLt, harness only) in front of every observation point; median of 5 x 6 steps
    calls3 = w3e.step_calls(0)
    tokens3 = int((calls3[0].reqs[:, 1] + calls3[0].reqs[:, 3] * calls3[0].reqs[:, 4]).max())
    x3 = calls3[0].tensor[:tokens3]
    w_mm = torch.randn(4096, 4096, device=dev).to(torch.bfloat16)
    y3 = torch.empty(tokens3, 4096, dtype=torch.bfloat16, device=dev)
    r3o = B.Ring(w3e.device_ring_bytes, w3e.host_ring_bytes, flags=B.BG_THREAD, max_reqs_per_observe=w3e.max_reqs)
    r3o.set_policy(w3e.policy_mode, 1, 0)
    p3 = [dmi.PreparedObserve(r3o, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype) for c in calls3]

    def prefill_steps(first, count, capture):
        for s3 in range(first, first + count):
            for po in p3:
                torch.matmul(x3, w_mm, out=y3)
                if capture:
                    ctx.check(po(s3, sh))
            if capture:
                ctx.consume(r3o)

    prefill_steps(0, 2, True)
    stream.synchronize()
    per3 = {False: [], True: []}
    for rep in range(5):
        for capture in (False, True):
            torch.cuda.synchronize()
            t = time.perf_counter()
            prefill_steps(10 + rep * 6, 6, capture)
            stream.synchronize()
            per3[capture].append((time.perf_counter() - t) * 1e3 / 6)
    ctx.settle(r3o)
    st3 = r3o.get_stats()
    r3o.destroy()
    b3, c3t = statistics.median(per3[False]), statistics.median(per3[True])
    extra["overhead_config3_prefill"] = {
        "no_capture_ms_per_step": round(b3, 3), "capture_ms_per_step": round(c3t, 3),
        "overhead_pct": round((c3t - b3) / b3 * 100, 3), "tokens_per_step": tokens3,
        "dropped_fraction": round(st3.dropped_bytes / max(1, st3.dropped_bytes + st3.captured_bytes), 4),
        "interfering_workload": f"10 x bf16 [{tokens3}, 4096] x [4096, 4096] matmul per step, one before each observe",
        "paper_context": "1.36 % prefill overhead on H100 (other hardware, real models)"}
    log(f"overhead, config 3 prefill: {extra['overhead_config3_prefill']}")
    del w3e, calls3, x3, y3, p3
    ctx.free()
    w4e = configs.config4_paged_kv(device=dev, n_steps=12)
    timed_replay("config4_paged_kv_12steps", w4e, block_timeout_ms=5000)
    timed_replay("config4_paged_kv_12steps_back_to_back", w4e, block_timeout_ms=5000, compute=False)
    timed_replay("config4_paged_kv_12steps_back_to_back_batched", w4e, block_timeout_ms=5000, compute=False, batch=8)
    del w4e
    ctx.free()
    extra["end_to_end"] = e2e


# ---------------------------------------------------------------------- front end, host cost
def run_hook_cost(ctx, extra):
    """Host microseconds per eager hook: the HookPoint module (custom operator), the binding's
    prepared call, and how long the foreign call alone takes, on the config-2 record."""
    dmi, B, configs, torch, dev, sh = ctx.dmi, ctx.B, ctx.configs, ctx.torch, ctx.dev, ctx.sh
    from paper_2605_11093_amd import hookpoint as hp
    wl = configs.config2_decode8b(device=dev, n_points=1, n_steps=1)
    c = wl.step_calls(0)[0]
    ring = B.Ring(1 << 30, 1 << 28, flags=B.BG_THREAD, max_reqs_per_observe=256)
    res = {}
    n = 2000
    po = dmi.PreparedObserve(ring, c.point_id, c.tensor, c.reqs, out_dtype=c.out_dtype, summary_mask=c.summary_mask)
    for i in range(200):
        ctx.check(po(i, sh))
    ctx.settle(ring)
    t = time.perf_counter()
    for i in range(n):
        po(i, sh)
        if i % 256 == 255:
            ctx.consume(ring)
    res["prepared_observe_us"] = round((time.perf_counter() - t) / n * 1e6, 2)
    ctx.settle(ring)
    sctx = hp.StepContext()
    hook = hp.HookPoint(ring, c.point_id, sctx, out_dtype=c.out_dtype, summary_mask=c.summary_mask)
    sctx.prepare_step(0, c.reqs)
    x = c.tensor
    with torch.no_grad():
        for i in range(200):
            hook(x)
        ctx.settle(ring)
        t = time.perf_counter()
        for i in range(n):
            hook(x)
            if i % 256 == 255:
                ctx.consume(ring)
        res["eager_hookpoint_us"] = round((time.perf_counter() - t) / n * 1e6, 2)
    ctx.settle(ring)
    ring.destroy()
    extra["host_us_per_hook"] = res
    log(f"host cost per hook: {res}")


# ---------------------------------------------------------------------- CPU oracle baseline
def run_cpu_baseline(ctx, budget_s=25.0):
    """The oracle's record builder, as it stands, on one host core over a prefix of the headline
    workload's records (config 5, hook order)."""
    import oracle
    from oracle.replay import CpuView
    oracle.build()
    w = ctx.configs.config5_saturation(device=ctx.dev, n_steps=4)
    calls = [w.step_calls(s) for s in range(4)]
    view = CpuView()
    t = time.perf_counter()
    nbytes = seq = steps = 0
    for s in range(200):
        for c in calls[s % 4]:
            rec = oracle.build_record(view.tensor(c.tensor), c.reqs, seq=seq, step_id=s, point_id=c.point_id,
                                      out_dtype=c.out_dtype, summary_mask=c.summary_mask)
            nbytes += rec.size
            seq += 1
        steps = s + 1
        if time.perf_counter() - t > budget_s:
            break
    dt = time.perf_counter() - t
    cpu = {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"record building for the first {steps} steps ({seq} records, {nbytes / 1e6:.0f} MB) of the "
                     f"same workload (config 5), {dt:.1f} s"}
    log(f"cpu oracle: {cpu}")
    del w, calls
    ctx.free()
    # the other configurations' records, a few seconds each (record bytes built per second, one core)
    others = {}
    for name, make in (("config1", lambda: ctx.configs.config1_tiny(device=ctx.dev)),
                       ("config2", lambda: ctx.configs.config2_decode8b(device=ctx.dev, n_steps=4)),
                       ("config3", lambda: ctx.configs.config3_prefill(device=ctx.dev, n_steps=1)),
                       ("config4", lambda: ctx.configs.config4_paged_kv(device=ctx.dev, n_steps=1, n_layers_cap=1))):
        w = make()
        view = CpuView()
        n_steps = w.n_steps
        pre = [w.step_calls(s) for s in range(min(n_steps, 4))]
        for cs in pre:                               # device -> host copies of the inputs are not the oracle's work
            for c in cs:
                view.tensor(c.tensor)
                view.paged(c.paged)
        t = time.perf_counter()
        nbytes = seq = 0
        rounds = 0
        while time.perf_counter() - t < 3.0 and rounds < 64:
            for cs in pre:
                for c in cs:
                    rec = oracle.build_record(view.tensor(c.tensor), c.reqs, seq=seq, step_id=0, point_id=c.point_id,
                                              out_dtype=c.out_dtype, summary_mask=c.summary_mask, keep_mask=c.keep_mask,
                                              row_index=c.row_index, paged=view.paged(c.paged))
                    nbytes += rec.size
                    seq += 1
                    if time.perf_counter() - t > 3.0:
                        break
                if time.perf_counter() - t > 3.0:
                    break
            rounds += 1
        dt = time.perf_counter() - t
        others[name] = {"GBs": round(nbytes / dt / 1e9, 4), "records": seq, "seconds": round(dt, 2)}
        del w, pre, view
        ctx.free()
    cpu["other_configs_record_GBs"] = others
    log(f"cpu oracle, other configurations: {others}")
    return cpu


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-overhead", action="store_true")
    ap.add_argument("--skip-extra", action="store_true")
    ap.add_argument("--profile-shape", default=None,
                    help="launch just this kernel shape (or a comma-separated list) a fixed number of times and "
                         "exit: the run rocprofv3 is pointed at.  'copy' adds a plain 256 MiB copy of known size, "
                         "the reference the profiler's HBM byte counters are scaled by; 'list' names the shapes")
    ap.add_argument("--kernels", default=None,
                    help="time just these kernel shapes (comma-separated names, see --profile-shape list) and exit")
    ap.add_argument("--hook-cost", action="store_true", help="measure just the host cost per hook and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build is a one-GPU path (each rank runs a private ring with no "
            "cross-GPU traffic); run with --gpus 1")
        sys.exit(2)

    ctx = Ctx()
    torch = ctx.torch
    if args.profile_shape:
        names = args.profile_shape.split(",")
        if "list" in names:
            for cfg, gen in shape_table(ctx).items():
                for name, *_ in gen():
                    print(name)
                ctx.free()
            return
        if "copy" in names:
            ca = torch.empty(256 << 20, dtype=torch.uint8, device=ctx.dev)
            cb = torch.empty_like(ca)
            for _ in range(3):
                ctx.bl.dmi_bench_copy(cb.data_ptr(), ca.data_ptr(), 256 << 20, ctx.sh)
            ctx.stream.synchronize()
            log("plain copy: 268435456 B read + 268435456 B written, 3 launches")
            del ca, cb
        run_kernel_table(ctx, only=[n for n in names if n != "copy"], profile=True)
        return

    if args.kernels:
        print(json.dumps(run_kernel_table(ctx, only=args.kernels.split(","))), flush=True)
        return

    extra = {}
    if args.hook_cost:
        run_hook_cost(ctx, extra)
        print(json.dumps(extra), flush=True)
        return
    run_probes(ctx, extra)

    # ------------------------------------------------------------------ headline: config 5, k = 1, batched
    c5 = Config5(ctx)
    base5 = c5.baseline()
    log(f"config 5: no-capture step {base5 * 1e3:.3f} ms")
    head = c5.run(1, "batched", args.steps, warmup=args.warmup, events=True)
    log(f"config 5 headline (k=1, batched): {head}")
    value, ms_per_step = head["delivered_GBs"], head["ms_per_step"]
    n_launch = head["launches"]
    alg_total = head["captured_records"] * Config5.ALG_PER_RECORD
    cap_us = head["launch_us_mean"]
    cap_gbs = alg_total / n_launch / cap_us / 1e3
    roofline = {"bound": "hbm",
                "kernel": "capture_kernel<bf16, 16-byte units, raw, no summaries>, one launch for the step's 80 "
                          "tensors (config 5), every launch of the headline's timed region",
                "timing": "HIP events that take the launch's own start and end time stamps from the hardware "
                          "(hipExtLaunchKernelGGL on the launch stream): the kernel's duration as a profiler reports it",
                "achieved": round(cap_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(cap_gbs / HBM_PEAK_GBS, 4), "us_per_launch": round(cap_us, 3),
                "us_per_launch_min": round(head["launch_us_min"], 3),
                "us_per_launch_max": round(head["launch_us_max"], 3), "launches": n_launch,
                "launches_timed": head["launches_timed"],
                "algorithmic_bytes_per_launch": round(alg_total / n_launch),
                "records_kept_per_launch": round(head["captured_records"] / n_launch, 2),
                # for comparison, markers recorded on the stream before and after the call, and the same
                # pair at the same place in a step with nothing between them
                "us_per_launch_between_events": round(head["launch_us_between_events_mean"], 3),
                "us_between_the_events_with_nothing_between": round(c5.empty_bracket_us, 3),
                # the profiled launch keeps all 80 records; a launch of this run kept this share of them
                "traffic": round(TRAFFIC_CONFIG5_BATCH80_BYTES * head["captured_records"] / n_launch / 80),
                "traffic_of_a_launch_that_keeps_all_80_records": TRAFFIC_CONFIG5_BATCH80_BYTES,
                "traffic_source": "profiles/hbm_traffic_counters.md"}
    log(f"roofline: {roofline}")
    sat = {}
    if not args.skip_extra:
        n5 = 100
        for mode in ("batched", "inline"):
            for k in (1, 2, 4, 8):
                r = c5.run(k, mode, n5, first_step=1000 * k)
                for drop in ("released_bytes", "captured_records", "dropped_records"):
                    r.pop(drop, None)
                sat[f"{mode}_k={k}"] = r
                log(f"config 5 saturation {mode} k={k}: {r}")
        sat["request_granular_drop_recent_batched"] = c5.request_granular(n5)
        log(f"config 5 saturation, request-granular best effort: {sat['request_granular_drop_recent_batched']}")
        extra["config5_saturation"] = {"no_capture_ms_per_step": round(base5 * 1e3, 3), "steps": n5,
                                       "interfering_workload": "80 x 219 MB bf16 weight-streaming GEMV per step",
                                       "runs": sat}
    c5.close()

    if not args.skip_extra:
        run_second_queue_probe(ctx, extra)
        extra["kernels"] = run_kernel_table(ctx)
    run_config2(ctx, extra, args.skip_overhead or args.skip_extra)
    if not args.skip_extra:
        run_configs34(ctx, extra)
        run_hook_cost(ctx, extra)
    cpu = None if args.skip_cpu_baseline else run_cpu_baseline(ctx)

    out = {
        "metric": "sustained captured GB/s to pinned host + % step-time overhead vs no-capture",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": SEED_NOTE,
        "config": {"workload": "config 5: saturation, Llama-70B-shaped decode, hidden 8192 bf16, 80 observation points, "
                               "256 requests x 1 row, raw bf16, device ring 4 GiB, host ring 16 GiB, policy "
                               "drop-newest, 1-in-k sampling with k = 1",
                   "bytes_per_captured_step": c5.rec_bytes * 80,
                   "dropped_fraction": head["dropped_fraction"],
                   "capture": "one batched launch per step (dmi_observe_batch over the step's 80 tensors)",
                   "model_stand_in": "80 x 219 MB bf16 weight-streaming GEMV per step (one GPU's TP-8 share of a 70B model); "
                                     "the host keeps at most two steps in flight, as a decode loop that waits for its "
                                     "sampled tokens does",
                   "drain": "copy engine, the library's drain thread; the producer thread polls and releases each step",
                   "timed_region": "steps plus delivery of everything captured (flush, poll, release)"},
        "frac_of_pinned_d2h_peak": round(value / ctx.d2h_peak, 3),
        "overhead_pct": head.get("overhead_pct"),
        "no_capture_ms_per_step": round(base5 * 1e3, 4),
        "ms_per_step_stream": head["ms_per_step_stream"],
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    out.update(extra)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
