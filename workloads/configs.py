"""Synthetic workloads shaped like the paper's LLM runs (evaluation setup:
Qwen3 / Llama-3.1 models on ShareGPT and WildChat-1M prompts).  Neither the
datasets nor any weights are used: the capture path is data-oblivious, so
seeded ~N(0,1) bf16 activations of the same shapes, ragged length mixes and
paged-cache structure stand in for them.

A workload is a list of steps; a step is a list of ObserveCall descriptors in
the order the hooks would fire.  Both the HIP path's driver and the CPU
oracle's driver consume these descriptors; nothing here gathers, converts or
packs anything.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional

import numpy as np
import torch

from . import prng

# dtype / policy codes are plain numbers in both the C ABI and the oracle.
DT_NONE, DT_BF16, DT_FP16, DT_FP32, DT_FP8 = 0, 1, 2, 3, 4
SUM_L2, SUM_MEAN, SUM_ABSMAX = 1, 2, 4
POLICY_BLOCK, POLICY_DROP_NEWEST = 0, 1

REQ_FIELDS = ("req_id", "row_base", "tok_start", "tok_count", "tok_step")


def make_reqs(rows) -> np.ndarray:
    """rows: iterable of (req_id, row_base, tok_start, tok_count, tok_step)."""
    a = np.asarray(list(rows), dtype=np.uint32).reshape(-1, 5)
    return np.ascontiguousarray(a)


@dataclass
class PagedSpec:
    block_size: int
    n_heads: int
    head_dim: int
    heads_sel: List[int]
    block_table: torch.Tensor          # int32 [n_seqs, max_blocks], workload device


@dataclass
class ObserveCall:
    point_id: int
    step_id: int
    tensor: torch.Tensor               # dense: [T, E] (row stride may exceed E); paged: [blocks, slots, heads, dim]
    reqs: np.ndarray                   # uint32 [n_reqs, 5], see REQ_FIELDS
    out_dtype: int = DT_BF16
    summary_mask: int = 0
    keep_mask: Optional[np.ndarray] = None    # uint8 [n_reqs]
    row_index: Optional[np.ndarray] = None    # int32, request-major explicit rows
    paged: Optional[PagedSpec] = None


@dataclass
class Workload:
    name: str
    device_ring_bytes: int
    host_ring_bytes: int
    policy_mode: int
    sample_k: int
    n_steps: int
    step_calls: Callable[[int], List[ObserveCall]]
    max_reqs: int = 256
    notes: Dict[str, object] = field(default_factory=dict)

    def steps(self):
        for s in range(self.n_steps):
            yield s, self.step_calls(s)


def _pool(seed_tags, n_slots, shape, device):
    """n_slots independent bf16 tensors of one shape."""
    n = int(np.prod(shape))
    return [prng.randn_bf16(prng.sub_seed(*seed_tags, s), n, device).view(*shape)
            for s in range(n_slots)]


# --------------------------------------------------------------------------
# config 1: tiny
# --------------------------------------------------------------------------
def tiny_lengths(step: int, n_reqs: int = 4, lo: int = 1, hi: int = 17,
                 cap: int = 64) -> np.ndarray:
    """Ragged lengths uniform in [lo, hi]; while the total exceeds `cap` the
    currently longest request (lowest index on ties) loses one token."""
    lens = prng.randint(prng.sub_seed(1, 7, step), n_reqs, lo, hi)
    while lens.sum() > cap:
        lens[int(np.argmax(lens))] -= 1
    return lens


def config1_tiny(device="cpu", n_points=8, n_steps=16, hidden=256,
                 device_ring_bytes=1 << 20, host_ring_bytes=4 << 20) -> Workload:
    pools = [_pool((1, p), 4, (64, hidden), device) for p in range(n_points)]

    def step_calls(step):
        lens = tiny_lengths(step)
        base = np.concatenate([[0], np.cumsum(lens)[:-1]])
        reqs = make_reqs((1000 + r, int(base[r]), int(lens[r]) - 1, 1, 1)
                         for r in range(len(lens)))
        return [ObserveCall(point_id=p, step_id=step, tensor=pools[p][step % 4],
                            reqs=reqs, out_dtype=DT_BF16) for p in range(n_points)]

    return Workload("tiny", device_ring_bytes, host_ring_bytes, POLICY_BLOCK, 1,
                    n_steps, step_calls, max_reqs=64)


# --------------------------------------------------------------------------
# config 2 / 5: decode, one row per request at every layer
# --------------------------------------------------------------------------
def _decode(name, tag, device, hidden, n_points, n_reqs, n_steps, summary_mask,
            device_ring_bytes, host_ring_bytes, policy_mode, sample_k) -> Workload:
    pools = [_pool((tag, p), 4, (n_reqs, hidden), device) for p in range(n_points)]

    def step_calls(step):
        reqs = make_reqs((5000 + r, r, 0, 1, 1) for r in range(n_reqs))
        return [ObserveCall(point_id=p, step_id=step, tensor=pools[p][step % 4],
                            reqs=reqs, out_dtype=DT_BF16, summary_mask=summary_mask)
                for p in range(n_points)]

    return Workload(name, device_ring_bytes, host_ring_bytes, policy_mode, sample_k,
                    n_steps, step_calls, max_reqs=max(64, n_reqs))


def config2_decode8b(device="cpu", n_points=32, n_reqs=64, n_steps=256, hidden=4096,
                     device_ring_bytes=256 << 20, host_ring_bytes=2 << 30) -> Workload:
    return _decode("decode8b", 2, device, hidden, n_points, n_reqs, n_steps,
                   SUM_L2 | SUM_ABSMAX, device_ring_bytes, host_ring_bytes,
                   POLICY_BLOCK, 1)


def config5_saturation(device="cpu", n_points=80, n_reqs=256, n_steps=200, hidden=8192,
                       sample_k=1, device_ring_bytes=4 << 30,
                       host_ring_bytes=16 << 30) -> Workload:
    return _decode("saturation70b", 5, device, hidden, n_points, n_reqs, n_steps, 0,
                   device_ring_bytes, host_ring_bytes, POLICY_DROP_NEWEST, sample_k)


# --------------------------------------------------------------------------
# config 3: ragged prefill, every 4th token, fp8 downcast
# --------------------------------------------------------------------------
def config3_prefill(device="cpu", n_reqs=32, len_lo=128, len_hi=2048, n_steps=8,
                    hidden=4096, inter=14336, n_resid=8, n_mlp=2, tok_step=4,
                    out_dtype=DT_FP8, device_ring_bytes=512 << 20,
                    host_ring_bytes=4 << 30) -> Workload:
    t_max = n_reqs * len_hi
    resid = [prng.randn_bf16(prng.sub_seed(3, 0, p), t_max * hidden, device).view(t_max, hidden)
             for p in range(n_resid)]
    mlp = [prng.randn_bf16(prng.sub_seed(3, 1, p), t_max * inter, device).view(t_max, inter)
           for p in range(n_mlp)]

    def step_calls(step):
        lens = prng.randint(prng.sub_seed(3, 9, step), n_reqs, len_lo, len_hi)
        base = np.concatenate([[0], np.cumsum(lens)[:-1]])
        reqs = make_reqs((7000 + 100 * step + r, int(base[r]), 0,
                          -(-int(lens[r]) // tok_step), tok_step) for r in range(n_reqs))
        calls = []
        # hook order inside a layer stack: residual points interleaved with the MLP ones
        mlp_after = {max(0, n_resid // 2 - 1): 0, n_resid - 1: 1} if n_mlp == 2 else \
                    {i: i for i in range(n_mlp)}
        for p in range(n_resid):
            calls.append(ObserveCall(point_id=p, step_id=step, tensor=resid[p], reqs=reqs,
                                     out_dtype=out_dtype))
            if p in mlp_after and mlp_after[p] < n_mlp:
                m = mlp_after[p]
                calls.append(ObserveCall(point_id=100 + m, step_id=step, tensor=mlp[m],
                                         reqs=reqs, out_dtype=out_dtype))
        return calls

    return Workload("prefill_ragged", device_ring_bytes, host_ring_bytes,
                    POLICY_DROP_NEWEST, 1, n_steps, step_calls, max_reqs=max(64, n_reqs))


# --------------------------------------------------------------------------
# config 4: paged KV-cache slices
# --------------------------------------------------------------------------
def config4_paged_kv(device="cpu", n_layers_cap=4, n_blocks=65536, block_size=16,
                     n_heads=8, head_dim=128, n_reqs=128, ctx_lo=512, ctx_hi=8192,
                     reqs_per_step=16, n_steps=128, heads_sel=(1, 5),
                     device_ring_bytes=2 << 30, host_ring_bytes=8 << 30) -> Workload:
    ctx0 = prng.randint(prng.sub_seed(4, 1), n_reqs, ctx_lo, ctx_hi)
    need = -(-(ctx0 + n_steps) // block_size)            # blocks per request
    max_blocks = int(-(-(ctx_hi + n_steps) // block_size))
    assert int(need.sum()) <= n_blocks, "context mix does not fit the physical block pool"
    perm = prng.permutation(prng.sub_seed(4, 2), n_blocks)
    table = np.full((n_reqs, max_blocks), -1, dtype=np.int32)
    cur = 0
    for r in range(n_reqs):
        table[r, :need[r]] = perm[cur:cur + need[r]]
        cur += int(need[r])
    # unused entries point at a valid block so that no selection can leave the cache
    table[table < 0] = 0
    block_table = torch.from_numpy(table).to(device)
    shape = (n_blocks, block_size, n_heads, head_dim)
    n = int(np.prod(shape))
    caches = [[prng.randn_bf16(prng.sub_seed(4, 3, l, kv), n, device).view(*shape)
               for kv in range(2)] for l in range(n_layers_cap)]
    spec = PagedSpec(block_size, n_heads, head_dim, list(heads_sel), block_table)

    def step_calls(step):
        chosen = np.sort(prng.permutation(prng.sub_seed(4, 5, step), n_reqs)[:reqs_per_step])
        reqs = make_reqs((9000 + int(r), int(r), 0, int(ctx0[r]) + step, 1) for r in chosen)
        return [ObserveCall(point_id=2 * l + kv, step_id=step, tensor=caches[l][kv],
                            reqs=reqs, out_dtype=DT_BF16, paged=spec)
                for l in range(n_layers_cap) for kv in range(2)]

    return Workload("paged_kv", device_ring_bytes, host_ring_bytes, POLICY_BLOCK, 1,
                    n_steps, step_calls, max_reqs=max(64, reqs_per_step),
                    notes={"ctx0": ctx0, "layers": [0, 10, 21, 31][:n_layers_cap]})


# --------------------------------------------------------------------------
# replayed step: the same list of observes every step (fixed tensor shapes, request
# counts and transforms, as a captured graph has them), while tensor contents, batch
# composition, keep vectors, row indices and block tables change from step to step
# --------------------------------------------------------------------------
def replayed_step(n_steps=6, n_graph=6, eager_extra_every=0, policy_mode=POLICY_BLOCK, sample_k=1,
                  device_ring_bytes=4 << 20, host_ring_bytes=16 << 20) -> Workload:
    """Host-side workload (tensors on the CPU; a harness copies each step's contents
    into its static device buffers).  The first `n_graph` calls of every step are the
    step's fixed launches, in a fixed order:
      0  bf16 [64, 1024]   one row per request in rows 0..63, raw + L2 + absmax
      1  bf16 [64, 1024]   same selection, fp8 out
      2  bf16 [300, 256]   ragged token ranges + keep vector, fp16 out, mean
      3  fp32 [40, 101]    explicit row indices (rows not 16-byte movable), raw
      4  bf16 paged [48, 16, 4, 64], heads {1, 3}, token ranges that grow, raw + absmax
      5  bf16 [64, 1024]   one row per request, rows permuted per step, raw
    With eager_extra_every = m > 0 every m-th step ends with one more observe that
    is not part of the fixed list (issued the ordinary way between replays)."""
    assert 1 <= n_graph <= 6
    n_r = 64

    def t_bf16(tag, step, shape):
        return prng.randn_bf16(prng.sub_seed(9, tag, step), int(np.prod(shape))).view(*shape)

    block_size, n_heads, head_dim, n_blocks, n_seqs, max_blocks = 16, 4, 64, 48, 6, 8

    def step_calls(step):
        calls = []
        # 0, 1: decode-shaped, request ids change with the step
        reqs01 = make_reqs((100 * step + r, r, 0, 1, 1) for r in range(n_r))
        x0 = t_bf16(0, step, (n_r, 1024))
        calls.append(ObserveCall(point_id=0, step_id=step, tensor=x0, reqs=reqs01, out_dtype=DT_BF16,
                                 summary_mask=SUM_L2 | SUM_ABSMAX))
        calls.append(ObserveCall(point_id=1, step_id=step, tensor=t_bf16(1, step, (n_r, 1024)), reqs=reqs01,
                                 out_dtype=DT_FP8))
        # 2: ragged ranges inside 5 requests of 60 rows each, keep vector
        lens = prng.randint(prng.sub_seed(9, 20, step), 5, 0, 12)
        starts = prng.randint(prng.sub_seed(9, 21, step), 5, 0, 20)
        reqs2 = make_reqs((7 * step + r, 60 * r, int(starts[r]), int(lens[r]), 1 + (r + step) % 3)
                          for r in range(5))
        keep2 = (prng.randint(prng.sub_seed(9, 22, step), 5, 0, 3) > 0).astype(np.uint8)
        calls.append(ObserveCall(point_id=2, step_id=step, tensor=t_bf16(2, step, (300, 256)), reqs=reqs2,
                                 out_dtype=DT_FP16, summary_mask=SUM_MEAN, keep_mask=keep2))
        # 3: fp32, explicit rows (3 requests x 4 rows)
        rows3 = prng.randint(prng.sub_seed(9, 30, step), 12, 0, 39).astype(np.int32)
        reqs3 = make_reqs((50 + r, 0, 10 * step + r, 4, 2) for r in range(3))
        calls.append(ObserveCall(point_id=3, step_id=step, tensor=t_bf16(3, step, (40, 101)).float(),
                                 reqs=reqs3, out_dtype=DT_FP32, row_index=rows3))
        # 4: paged cache, contexts grow by one token per step, block table reshuffled per step
        table = prng.permutation(prng.sub_seed(9, 40, step), n_blocks).astype(np.int32).reshape(n_seqs, max_blocks)
        spec = PagedSpec(block_size, n_heads, head_dim, [1, 3], torch.from_numpy(np.ascontiguousarray(table)))
        reqs4 = make_reqs((900 + r, r + 1, 0, 20 + 9 * r + step, 1) for r in range(4))
        calls.append(ObserveCall(point_id=4, step_id=step,
                                 tensor=t_bf16(4, step, (n_blocks, block_size, n_heads, head_dim)),
                                 reqs=reqs4, out_dtype=DT_BF16, summary_mask=SUM_ABSMAX, paged=spec))
        # 5: one row per request, rows permuted
        perm = prng.permutation(prng.sub_seed(9, 50, step), n_r)
        reqs5 = make_reqs((3000 + r, int(perm[r]), 0, 1, 1) for r in range(n_r))
        calls.append(ObserveCall(point_id=5, step_id=step, tensor=t_bf16(5, step, (n_r, 1024)), reqs=reqs5,
                                 out_dtype=DT_BF16))
        calls = calls[:n_graph]
        if eager_extra_every and step % eager_extra_every == eager_extra_every - 1:
            reqs6 = make_reqs([(1, 2, 0, 3, 1)])
            calls.append(ObserveCall(point_id=6, step_id=step, tensor=x0, reqs=reqs6, out_dtype=DT_BF16))
        return calls

    return Workload("replayed_step", device_ring_bytes, host_ring_bytes, policy_mode, sample_k, n_steps,
                    step_calls, max_reqs=64, notes={"n_graph": n_graph})


def replayed_batches(n_steps=5, policy_mode=POLICY_BLOCK, sample_k=1, device_ring_bytes=8 << 20,
                     host_ring_bytes=32 << 20, eager_extra_every=0, long_rows=0) -> Workload:
    """Host-side workload for replayed steps whose hooks can share launches: every step lists,
    in hook order,
      0-4   five bf16 [64, 1024] tensors, one row per request (ids and rows change per step), raw + L2
      5-7   three bf16 [300, 256] tensors, ragged token ranges + one keep vector, fp8 out, absmax
      8-9   K and V of a paged cache [48, 16, 4, 64], heads {1, 3}, contexts that grow, raw
      10    one more bf16 [64, 1024] tensor with the selection of 0-4 but fp16 out (its own launch)
    Consecutive calls of a group have the same layout, selection and transform.
    long_rows = n > 0 adds, as points 12..12+n-1, n bf16 [2400, 2048] tensors with ragged token ranges of
    some 2,000 rows, fp8 out: rows of 4 KiB, enough of them that one launch for the group has more
    work than fits the GPU at once."""
    n_r = 64
    block_size, n_heads, head_dim, n_blocks, n_seqs, max_blocks = 16, 4, 64, 48, 6, 8

    def t_bf16(tag, step, shape):
        return prng.randn_bf16(prng.sub_seed(19, tag, step), int(np.prod(shape))).view(*shape)

    def step_calls(step):
        calls = []
        perm = prng.permutation(prng.sub_seed(19, 50, step), n_r)
        reqs_a = make_reqs((100 * step + r, int(perm[r]), 0, 1, 1) for r in range(n_r))
        for i in range(5):
            calls.append(ObserveCall(point_id=i, step_id=step, tensor=t_bf16(i, step, (n_r, 1024)), reqs=reqs_a,
                                     out_dtype=DT_BF16, summary_mask=SUM_L2))
        lens = prng.randint(prng.sub_seed(19, 20, step), 5, 0, 12)
        starts = prng.randint(prng.sub_seed(19, 21, step), 5, 0, 20)
        reqs_b = make_reqs((7 * step + r, 60 * r, int(starts[r]), int(lens[r]), 1 + (r + step) % 3) for r in range(5))
        keep_b = (prng.randint(prng.sub_seed(19, 22, step), 5, 0, 3) > 0).astype(np.uint8)
        for i in range(5, 8):
            calls.append(ObserveCall(point_id=i, step_id=step, tensor=t_bf16(i, step, (300, 256)), reqs=reqs_b,
                                     out_dtype=DT_FP8, summary_mask=SUM_ABSMAX, keep_mask=keep_b))
        table = prng.permutation(prng.sub_seed(19, 40, step), n_blocks).astype(np.int32).reshape(n_seqs, max_blocks)
        spec = PagedSpec(block_size, n_heads, head_dim, [1, 3], torch.from_numpy(np.ascontiguousarray(table)))
        reqs_c = make_reqs((900 + r, r + 1, 0, 20 + 9 * r + step, 1) for r in range(4))
        for i in range(8, 10):
            calls.append(ObserveCall(point_id=i, step_id=step,
                                     tensor=t_bf16(i, step, (n_blocks, block_size, n_heads, head_dim)),
                                     reqs=reqs_c, out_dtype=DT_BF16, paged=spec))
        calls.append(ObserveCall(point_id=10, step_id=step, tensor=t_bf16(10, step, (n_r, 1024)), reqs=reqs_a,
                                 out_dtype=DT_FP16))
        if long_rows:
            lens_d = prng.randint(prng.sub_seed(19, 60, step), 6, 300, 400)
            reqs_d = make_reqs((40 * step + r, 400 * r, int(step % 3), int(lens_d[r]), 1) for r in range(6))
            for i in range(long_rows):
                calls.append(ObserveCall(point_id=12 + i, step_id=step, tensor=t_bf16(12 + i, step, (2400, 2048)),
                                         reqs=reqs_d, out_dtype=DT_FP8))
        if eager_extra_every and step % eager_extra_every == eager_extra_every - 1:
            calls.append(ObserveCall(point_id=11, step_id=step, tensor=calls[0].tensor,
                                     reqs=make_reqs([(1, 2, 0, 3, 1)]), out_dtype=DT_BF16))
        return calls

    return Workload("replayed_batches", device_ring_bytes, host_ring_bytes, policy_mode, sample_k, n_steps,
                    step_calls, max_reqs=64, notes={"n_graph": 11 + long_rows})
