"""Batched captures (dmi_observe_batch, dmi_observe_paged_batch, dmi_step_observe_batch):
several observation points in one launch must give exactly the stream of the same observes
issued one by one.  The oracle knows nothing of batches: it builds the records of the single
calls, in hook order, and the batched HIP path is compared with that."""
import numpy as np
import pytest
import torch

import oracle as orc
from oracle.replay import run_workload
from workloads import configs, prng
from _util import compare_record, compare_streams

pytestmark = pytest.mark.gpu

DT_NONE, DT_BF16, DT_FP16, DT_FP32, DT_FP8 = 0, 1, 2, 3, 4
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def run_gpu(B):
    from paper_2605_11093_amd.replay import run_workload_gpu
    return run_workload_gpu


def _batch(B, tensors, reqs, *, points=None, out_dtype=None, summary_mask=0, keep_mask=None, row_index=None,
           paged=None, ring_bytes=1 << 23, poison=0xA5, policy=None):
    """One batched observe on a fresh, poisoned ring -> list of (gpu record, oracle record)."""
    reqs = np.asarray(reqs, dtype=np.uint32).reshape(-1, 5)
    n = len(tensors)
    points = list(range(10, 10 + n)) if points is None else points
    src_dt = {torch.bfloat16: 1, torch.float16: 2, torch.float32: 3}[tensors[0].dtype]
    od = src_dt if out_dtype is None else out_dtype
    with B.Ring(ring_bytes, ring_bytes, max_reqs_per_observe=2048) as ring:
        ring.debug_fill_rings(poison)
        if policy is not None:
            ring.set_policy(policy)
        s = torch.cuda.current_stream()
        km = None if keep_mask is None else torch.tensor(keep_mask, dtype=torch.uint8, device=DEV)
        ri = None if row_index is None else torch.tensor(row_index, dtype=torch.int32, device=DEV)
        rc, done = ring.observe_batch(points, tensors, reqs, step_id=21, stream=s.cuda_stream, out_dtype=od,
                                      summary_mask=summary_mask, keep_mask=km, row_index=ri, paged=paged)
        assert rc == B.OK and done == n
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host(256)
        assert [v.seq for v in views] == list(range(n))
        got = [v.bytes() for v in views]
        st = ring.get_stats()
        assert st.captured_records == n and st.launched_records == n and st.observed_calls == n
        s.synchronize()
    cpu_paged = None
    if paged is not None:
        cpu_paged = configs.PagedSpec(paged.block_size, paged.n_heads, paged.head_dim, paged.heads_sel,
                                      paged.block_table.cpu())
    out = []
    for i, t in enumerate(tensors):
        ref = orc.build_record(t.cpu(), reqs, seq=i, step_id=21, point_id=points[i], out_dtype=od,
                               summary_mask=summary_mask, keep_mask=keep_mask, row_index=row_index, paged=cpu_paged)
        out.append((got[i], ref))
    return out


def _tensors(seed, n, T, E, pitch=None, dtype=torch.bfloat16):
    pitch = pitch or E
    out = []
    for i in range(n):
        t = prng.randn_bf16(prng.sub_seed(seed, i), T * pitch, DEV).view(T, pitch)[:, :E]
        out.append(t.to(dtype) if dtype != torch.bfloat16 else t)
    return out


# ------------------------------------------------------------------ one batched call, every kernel path
@pytest.mark.parametrize("n", [1, 2, 7, 128])
def test_decode_shaped_batch(B, n):
    ts = _tensors(31, n, 16, 512)
    reqs = [(100 + r, r, 0, 1, 1) for r in range(16)]
    for got, ref in _batch(B, ts, reqs, summary_mask=5):
        compare_record(got, ref)
    for got, ref in _batch(B, ts, reqs):
        assert np.array_equal(got, ref)


def test_decode_shaped_batch_with_keep_vector_and_fp8(B):
    ts = _tensors(32, 9, 70, 1024)
    reqs = [(r, 69 - r, 0, 1, 1) for r in range(70)]
    mask = (np.arange(70) % 3 != 1).astype(np.uint8)
    for got, ref in _batch(B, ts, reqs, keep_mask=mask, out_dtype=DT_FP8, summary_mask=7):
        compare_record(got, ref)


@pytest.mark.parametrize("n,T,E", [(33, 256, 8192), (70, 128, 16384), (40, 230, 4096)])
def test_large_decode_shaped_batch_takes_the_general_kernel(B, n, T, E):
    """Beyond some eight thousand rows a decode-shaped batch goes through the general kernel, a
    workgroup per work item (rows of 1024 units, rows of two items, two rows per item)."""
    ts = _tensors(43, n, T, E)
    reqs = [(7000 + r, T - 1 - r, 0, 1, 1) for r in range(T)]
    res = _batch(B, ts, reqs, ring_bytes=(n + 2) * orc.record_bytes(T, T, E, 1, 0) // 64 * 64)
    for got, ref in res:
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("E,T", [(4096, 300), (256, 3000), (14336, 40), (8192, 256)])
@pytest.mark.parametrize("out_dtype", [DT_BF16, DT_FP8])
def test_general_kernel_batch_long_rows(B, E, T, out_dtype):
    ts = _tensors(33, 3, T, E)
    reqs = [(1, 0, 0, T // 3, 2), (2, 2 * (T // 3), 1, T // 4, 1), (3, T - 1, 0, 1, 1)]
    # a keep vector with several rows per request keeps the launch on the general kernel
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, keep_mask=[1, 1, 1], ring_bytes=1 << 25):
        assert np.array_equal(got, ref)
    # without one, selections of up to 1024 rows take the decode-shaped kernel (a row map behind the table)
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, ring_bytes=1 << 25):
        assert np.array_equal(got, ref)


# A batch of long rows with more work items than fit the GPU at once: workgroups of a few items
# each, many more of them than are resident, tensor after tensor.
@pytest.mark.parametrize("E,T,n", [(4096, 3000, 4), (14336, 420, 3), (2048, 2600, 3), (5000, 700, 5), (4096, 1500, 128)])
@pytest.mark.parametrize("out_dtype", [DT_BF16, DT_FP8])
def test_long_batch_of_long_rows(B, E, T, n, out_dtype):
    if n == 128:
        T, per = 40, 11             # many small tensors: 128 x 40 rows of 512 units = 2,560 items
        ts = _tensors(35, n, T, E)
        reqs = [(1, 0, 0, per, 2), (2, 20, 1, 9, 2), (3, T - 1, 0, 1, 1)]
    else:
        ts = _tensors(35, n, T, E)
        q = T // 4
        reqs = [(1, 0, 0, q // 2, 2), (2, q, 3, q - 5, 1), (3, 2 * q, 0, q, 1), (4, 3 * q, 1, q // 3, 3), (5, T - 1, 0, 1, 1)]
    rows = sum(r[3] for r in reqs)
    es = 1 if out_dtype == DT_FP8 else 2
    ring = 1 << max(23, int(np.ceil(np.log2(n * (rows * E * es + 4096)))) + 1)
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, keep_mask=[1] * len(reqs), ring_bytes=ring):
        assert np.array_equal(got, ref)
    keep = [1, 0, 1, 1, 0][:len(reqs)]
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, keep_mask=keep, ring_bytes=ring):
        assert np.array_equal(got, ref)


def test_long_batch_of_long_rows_wraps_and_drops_mid_batch(B):
    """The same with the ring's end inside the batch, and under best effort with room for two and a
    half of four records: records 0 and 1 stay, 2 and 3 are dropped and counted."""
    E, T, n = 4096, 1600, 4
    ts = _tensors(36, n, T, E)
    reqs = np.array([(1, 0, 0, 700, 2), (2, 1400, 0, 200, 1), (3, 3, 0, 1, 1)], dtype=np.uint32)
    rb = orc.record_bytes(3, 901, E, DT_FP8, 0)
    km = torch.ones(3, dtype=torch.uint8, device=DEV)
    refs = [orc.build_record(t.cpu(), reqs, seq=0, step_id=0, point_id=0, out_dtype=DT_FP8, keep_mask=[1, 1, 1]) for t in ts]

    def same(v, i, seq, step, point):
        got, ref = v.bytes(), refs[i].copy()
        ref[8:16] = np.frombuffer(np.uint64(seq).tobytes(), dtype=np.uint8)
        ref[16:24] = np.frombuffer(np.uint64(step).tobytes(), dtype=np.uint8)
        ref[24:28] = np.frombuffer(np.uint32(point).tobytes(), dtype=np.uint8)
        assert np.array_equal(got, ref), (seq, i)

    s = torch.cuda.current_stream()
    # (a) completeness policy, ring of 4.6 records: the second batch starts at 4 records and wraps
    with B.Ring((rb * 46 // 10) // 64 * 64, 1 << 25) as ring:
        for step in range(3):
            rc, done = ring.observe_batch([5, 6, 7, 8], ts, reqs, step_id=step, stream=s.cuda_stream, out_dtype=DT_FP8,
                                          keep_mask=km)
            assert rc == B.OK and done == 4
            ring.drain(B.DRAIN_FLUSH)
            views = ring.poll_host()
            assert [v.seq for v in views] == [4 * step + i for i in range(4)]
            for i, v in enumerate(views):
                same(v, i, 4 * step + i, step, 5 + i)
            ring.release_host(views[-1].seq)
        assert ring.get_stats().dropped_records == 0
    # (b) best effort, ring of 2.5 records
    with B.Ring((rb * 5 // 2) // 64 * 64, 1 << 25) as ring:
        ring.set_policy(B.POLICY_DROP_NEWEST)
        for step in range(2):
            ring.observe_batch([5, 6, 7, 6], ts, reqs, step_id=step, stream=s.cuda_stream, out_dtype=DT_FP8, keep_mask=km)
            s.synchronize()
            ring.drain(B.DRAIN_FLUSH)
            views = ring.poll_host()
            assert [v.seq for v in views] == [4 * step, 4 * step + 1]
            for i, v in enumerate(views):
                same(v, i, 4 * step + i, step, 5 + i)
            ring.release_host(views[-1].seq)
        st = ring.get_stats()
        assert (st.captured_records, st.dropped_records, st.dropped_rows, st.dropped_bytes) == (4, 4, 4 * 901, 4 * rb)
        assert {p: ring.get_point_drops(p) for p in (5, 6, 7)} == {5: 0, 6: 2, 7: 2}


def test_long_paged_batch_of_long_rows(B):
    NB, BS, NH, HD = 80, 16, 8, 256              # rows of 8 heads x 256 = 2048 elements
    caches = [prng.randn_bf16(prng.sub_seed(39, i), NB * BS * NH * HD, DEV).view(NB, BS, NH, HD) for i in range(6)]
    table = torch.from_numpy(prng.permutation(4, NB).astype(np.int32).reshape(5, 16)).to(DEV)
    spec = configs.PagedSpec(BS, NH, HD, [7, 0, 3, 1, 2, 6, 5, 4], table)
    reqs = [(1, 2, 0, 256, 1), (2, 0, 5, 80, 3), (3, 3, 255, 1, 1), (4, 1, 0, 250, 1), (5, 4, 1, 255, 1), (6, 0, 0, 256, 1)]
    for got, ref in _batch(B, caches, reqs, paged=spec, ring_bytes=1 << 26):
        assert np.array_equal(got, ref)
    for got, ref in _batch(B, caches, reqs, paged=spec, keep_mask=[1, 1, 0, 1, 1, 1], out_dtype=DT_FP8, ring_bytes=1 << 26):
        assert np.array_equal(got, ref)


def test_empty_and_degenerate_batches(B):
    """Nothing to capture is still a well-formed answer: a batch of no tensors does nothing; a batch whose
    selection lists no request, or only requests without rows, or whose keep vector keeps nobody, gives
    one record per tensor with a header, a table and no rows, as the single observes do."""
    ts = _tensors(44, 3, 40, 256)
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream()
        import ctypes as C
        ra = np.array([(1, 0, 0, 1, 1)], dtype=np.uint32)
        like = B.Tensor(None, 1, (C.c_int64 * 2)(40, 256), (C.c_int64 * 2)(256, 1))
        sel, xf, done = B.Selection(1, ra.ctypes.data, None, None), B.Transform(1, 0), C.c_uint32(7)
        rc = B.lib().dmi_observe_batch(ring._h, 0, None, None, C.byref(like), C.byref(sel), C.byref(xf), 0,
                                       s.cuda_stream, C.byref(done))
        assert (rc, done.value) == (B.OK, 0) and ring.get_stats().launched_records == 0
    for reqs, km, sm in [(np.zeros((0, 5), np.uint32), None, 0),
                         ([(5, 3, 0, 0, 1), (6, 9, 2, 0, 4)], None, 7),
                         ([(1, 0, 0, 2, 1), (2, 7, 0, 3, 1)], [0, 0], 5)]:
        for got, ref in _batch(B, ts, reqs, keep_mask=km, summary_mask=sm):
            assert np.array_equal(got, ref)
        for got, ref in _batch(B, ts, reqs, keep_mask=km, out_dtype=DT_FP8):
            assert np.array_equal(got, ref)


@pytest.mark.parametrize("seed", range(48))
def test_random_batches_equal_the_oracles_single_records(B, seed):
    """A seeded sweep over what a batched call can be given: row widths on both sides of every path's
    limits (16-byte movable or not), tensor counts, ragged selections with empty requests, repeated and
    strided tokens, keep vectors, every transform, row pitches wider than the rows."""
    rng = np.random.RandomState(1000 + seed)
    E = int(rng.choice([8, 56, 64, 250, 256, 264, 512, 1000, 1024, 2048, 2056, 4096, 5000, 8192, 9000]))
    T = int(rng.randint(1, 260)) if E <= 4096 else int(rng.randint(1, 60))
    n = int(rng.choice([1, 2, 3, 5, 9, 17]))
    pitch = E + int(rng.choice([0, 0, 8, 24])) if E % 8 == 0 else E
    ts = _tensors(500 + seed, n, T, E, pitch=pitch)
    n_reqs = int(rng.randint(1, 24))
    reqs = []
    for q in range(n_reqs):
        step = int(rng.choice([0, 1, 1, 1, 2, 3, 7]))
        count = int(rng.choice([0, 1, 1, 2, 5, 30]))
        base = int(rng.randint(0, T))
        start = int(rng.randint(0, T - base))
        if count > 1 and step > 0:
            count = min(count, (T - 1 - base - start) // step + 1)
        reqs.append((1000 + q, base, start, max(count, 0), step))
    keep = None
    if rng.rand() < 0.5:
        keep = [int(x) for x in (rng.rand(n_reqs) < 0.7)]
    out_dtype = int(rng.choice([DT_BF16, DT_BF16, DT_FP8, DT_FP16, DT_NONE]))
    sm = int(rng.randint(0, 8))
    if out_dtype == DT_NONE and sm == 0:
        sm = 5
    if out_dtype == DT_NONE and (sm & 2):
        sm |= 1                 # the mean's tolerance is scaled by the row's L2 when there is no payload
    rows = sum(r[3] for r in reqs)
    ring = 1 << max(22, int(np.ceil(np.log2(n * (rows * E * 2 + 64 * n_reqs + 8192)))) + 1)
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, summary_mask=sm, keep_mask=keep, ring_bytes=ring):
        compare_record(got, ref, what=f"seed {seed}: E={E} T={T} n={n} reqs={n_reqs} out={out_dtype} sm={sm}")


@pytest.mark.parametrize("seed", range(16))
def test_random_indexed_batches(B, seed):
    """The same sweep with an explicit row for every listed row (row_index_dev)."""
    rng = np.random.RandomState(3000 + seed)
    E = int(rng.choice([64, 256, 512, 1024, 4096, 8192]))
    T = int(rng.randint(4, 200))
    n = int(rng.choice([1, 2, 4, 9]))
    ts = _tensors(700 + seed, n, T, E)
    n_reqs = int(rng.randint(1, 20))
    reqs = [(50 + q, 0, int(rng.randint(0, 5)), int(rng.choice([0, 1, 1, 2, 6])), 1) for q in range(n_reqs)]
    listed = sum(r[3] for r in reqs)
    idx = rng.randint(0, T, size=max(listed, 1))[:listed]
    keep = [int(x) for x in (rng.rand(n_reqs) < 0.7)] if rng.rand() < 0.5 else None
    out_dtype = int(rng.choice([DT_BF16, DT_FP8, DT_FP16]))
    sm = int(rng.choice([0, 0, 1, 4, 5, 7]))
    for got, ref in _batch(B, ts, reqs, out_dtype=out_dtype, summary_mask=sm, keep_mask=keep, row_index=idx,
                           ring_bytes=1 << 24):
        compare_record(got, ref, what=f"seed {seed}: E={E} T={T} n={n} reqs={n_reqs} out={out_dtype} sm={sm}")


@pytest.mark.parametrize("seed", range(24))
def test_random_paged_batches(B, seed):
    """A seeded sweep over paged caches: block sizes, head counts and widths (rows of 64 bytes to 4 KiB), head
    subsets in any order, shuffled block tables, contexts that end anywhere in a block."""
    rng = np.random.RandomState(5000 + seed)
    BS = int(rng.choice([4, 8, 16, 32]))
    NH = int(rng.choice([1, 2, 4, 8]))
    HD = int(rng.choice([32, 64, 128, 256]))
    n_seqs, max_blocks = int(rng.randint(1, 6)), int(rng.randint(1, 9))
    NBLK = n_seqs * max_blocks + int(rng.randint(0, 8))
    n = int(rng.choice([1, 2, 4, 6]))
    caches = [prng.randn_bf16(prng.sub_seed(900 + seed, i), NBLK * BS * NH * HD, DEV).view(NBLK, BS, NH, HD) for i in range(n)]
    table = rng.permutation(NBLK)[:n_seqs * max_blocks].astype(np.int32).reshape(n_seqs, max_blocks)
    k = int(rng.randint(1, NH + 1))
    heads = [int(h) for h in rng.permutation(NH)[:k]]
    spec = configs.PagedSpec(BS, NH, HD, heads, torch.from_numpy(table).to(DEV))
    ctx_len = BS * max_blocks
    reqs = []
    for q in range(int(rng.randint(1, 12))):
        step = int(rng.choice([1, 1, 2, 5]))
        start = int(rng.randint(0, ctx_len))
        count = int(rng.choice([0, 1, 3, 40, 400]))
        if count:
            count = min(count, (ctx_len - 1 - start) // step + 1)
        reqs.append((70 + q, int(rng.randint(0, n_seqs)), start, count, step))
    keep = [int(x) for x in (rng.rand(len(reqs)) < 0.7)] if rng.rand() < 0.4 else None
    out_dtype = int(rng.choice([DT_BF16, DT_BF16, DT_FP8, DT_FP16]))
    sm = int(rng.choice([0, 0, 0, 1, 5, 7]))
    for got, ref in _batch(B, caches, reqs, paged=spec, out_dtype=out_dtype, summary_mask=sm, keep_mask=keep,
                           ring_bytes=1 << 25):
        compare_record(got, ref, what=f"seed {seed}: BS={BS} NH={NH} HD={HD} heads={heads} n={n} out={out_dtype} sm={sm}")


def test_general_kernel_batch_with_summaries_masks_and_indices(B):
    ts = _tensors(34, 5, 300, 512)
    reqs = [(10 + i, 20 * i, 0, 3 + i, 2) for i in range(9)]
    mask = [1, 0, 1, 1, 0, 0, 1, 0, 1]
    n = sum(r[3] for r in reqs)
    idx = (np.arange(n) * 37 + 11) % 300
    for got, ref in _batch(B, ts, reqs, keep_mask=mask, summary_mask=7):
        compare_record(got, ref)
    for got, ref in _batch(B, ts, reqs, row_index=idx, keep_mask=mask, out_dtype=DT_FP16):
        assert np.array_equal(got, ref)
    for got, ref in _batch(B, ts, reqs, keep_mask=[0] * 9):
        assert np.array_equal(got, ref) and got.size == 64 + 192


@pytest.mark.parametrize("E", [3, 250, 2056])
def test_batch_of_rows_that_are_not_16_byte_movable(B, E):
    ts = _tensors(35, 4, 37, E, pitch=E + 24)
    # one of the tensors sits at an odd element offset: the whole batch takes the element-wise kernel
    buf = prng.randn_bf16(36, 37 * (E + 24) + 8, DEV)
    ts[2] = buf[1: 1 + 37 * (E + 24)].view(37, E + 24)[:, :E]
    reqs = [(1, 0, 2, 3, 1), (2, 10, 0, 6, 4), (3, 36, 0, 1, 1), (4, 5, 0, 0, 1)]
    for got, ref in _batch(B, ts, reqs, summary_mask=2):
        compare_record(got, ref)


def test_fp32_batch(B):
    ts = _tensors(37, 3, 40, 512, dtype=torch.float32)
    for got, ref in _batch(B, ts, [(1, 3, 1, 9, 2), (2, 30, 0, 10, 1)], summary_mask=7):
        compare_record(got, ref)


def test_paged_batch(B):
    NB, BS, NH, HD = 64, 16, 8, 128
    caches = [prng.randn_bf16(prng.sub_seed(38, i), NB * BS * NH * HD, DEV).view(NB, BS, NH, HD) for i in range(4)]
    table = torch.from_numpy(prng.permutation(3, NB).astype(np.int32).reshape(4, 16)).to(DEV)
    spec = configs.PagedSpec(BS, NH, HD, [1, 5], table)
    reqs = [(1, 2, 0, 200, 1), (2, 0, 5, 40, 3), (3, 3, 255, 1, 1)]
    for got, ref in _batch(B, caches, reqs, paged=spec):
        assert np.array_equal(got, ref)
    for got, ref in _batch(B, caches, reqs, paged=spec, keep_mask=[0, 1, 1], summary_mask=5, out_dtype=DT_FP8):
        compare_record(got, ref)


def test_batch_larger_than_one_launch_and_mixed_layout_is_refused(B):
    ts = _tensors(39, 131, 4, 64)                     # 131 tensors: two launches (128 + 3)
    reqs = [(1, 0, 0, 2, 1), (2, 3, 0, 1, 1)]
    res = _batch(B, ts, reqs, points=[p % 4096 for p in range(500, 631)])
    assert len(res) == 131
    for got, ref in res:
        assert np.array_equal(got, ref)
    with pytest.raises(ValueError):
        with B.Ring(1 << 20, 1 << 20) as ring:
            ring.observe_batch([1, 2], [ts[0], _tensors(40, 1, 4, 128)[0]], reqs, step_id=0)


# ------------------------------------------------------------------ policy inside a batch
def test_disabled_points_and_sampling_inside_a_batch(B):
    ts = _tensors(41, 6, 8, 256)
    reqs = np.array([(r, r, 0, 1, 1) for r in range(8)], dtype=np.uint32)
    pts = [3, 4, 5, 6, 7, 8]
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream().cuda_stream
        ring.point_enable(4, False)
        ring.point_enable(8, False)
        rc, done = ring.observe_batch(pts, ts, reqs, step_id=0, stream=s)
        assert rc == B.OK and done == 6
        ring.set_policy(B.POLICY_BLOCK, 2, 0)
        rc, done = ring.observe_batch(pts, ts, reqs, step_id=1, stream=s)     # sampled out
        assert rc == B.SAMPLED_OUT and done == 6
        for p in (3, 5, 6, 7):
            ring.point_enable(p, False)
        rc, done = ring.observe_batch(pts, ts, reqs, step_id=2, stream=s)     # nothing enabled
        assert rc == B.POINT_DISABLED and done == 6
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert [v.seq for v in views] == [0, 1, 2, 3]
        for v, i in zip(views, (0, 2, 3, 4)):
            ref = orc.build_record(ts[i].cpu(), reqs, seq=v.seq, step_id=0, point_id=pts[i], out_dtype=1)
            assert np.array_equal(v.bytes(), ref)
        st = ring.get_stats()
        assert st.observed_calls == 18 and st.launched_records == 4 and st.captured_records == 4
        assert st.disabled_calls == 2 + 2 + 6 and st.sampled_out_calls == 4 and st.sampled_out_rows == 32


def test_drop_newest_in_the_middle_of_a_batch(B):
    """Ring of 5.5 records, batch of 8: records 0..4 stay, 5..7 are dropped and counted per point;
    a second batch with the ring still full drops everything; after a drain it is admitted again."""
    ts = _tensors(42, 8, 16, 512)
    reqs = np.array([(r, r, 0, 1, 1) for r in range(16)], dtype=np.uint32)
    rb = orc.record_bytes(16, 16, 512, 1, 0)
    pts = [20, 21, 22, 23, 24, 25, 26, 25]
    with B.Ring(rb * 5 + rb // 2 // 64 * 64, 1 << 22) as ring:
        ring.set_policy(B.POLICY_DROP_NEWEST)
        s = torch.cuda.current_stream()
        ring.observe_batch(pts, ts, reqs, step_id=0, stream=s.cuda_stream)
        ring.observe_batch(pts, ts, reqs, step_id=1, stream=s.cuda_stream)
        s.synchronize()
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert [v.seq for v in views] == [0, 1, 2, 3, 4]
        ring.release_host(4)
        ring.observe_batch(pts[:3], ts[:3], reqs, step_id=2, stream=s.cuda_stream)
        s.synchronize()
        ring.drain(B.DRAIN_FLUSH)
        more = ring.poll_host()
        assert [v.seq for v in more] == [16, 17, 18]
        for v in views:
            ref = orc.build_record(ts[v.seq].cpu(), reqs, seq=v.seq, step_id=0, point_id=pts[v.seq], out_dtype=1)
            assert np.array_equal(v.bytes(), ref)
        for v in more:
            i = v.seq - 16
            ref = orc.build_record(ts[i].cpu(), reqs, seq=v.seq, step_id=2, point_id=pts[i], out_dtype=1)
            assert np.array_equal(v.bytes(), ref)
        st = ring.get_stats()
        assert (st.captured_records, st.dropped_records) == (8, 11)
        assert (st.dropped_rows, st.dropped_bytes) == (11 * 16, 11 * rb)
        drops = {p: ring.get_point_drops(p) for p in set(pts)}
        assert drops == {20: 1, 21: 1, 22: 1, 23: 1, 24: 1, 25: 4, 26: 2}


@pytest.mark.parametrize("room", [1, 2, 7])
def test_drop_newest_keeps_a_prefix_of_any_length(B, room):
    """Room for `room` and a half records, batches of 8 decode-shaped tensors: exactly the first `room`
    stay (one kept record is a launch of its own kind: it would take the decode-shaped kernel if it
    did not also have to count the seven behind it)."""
    ts = _tensors(43, 8, 16, 1024)
    reqs = np.array([(r, 15 - r, 0, 1, 1) for r in range(16)], dtype=np.uint32)
    rb = orc.record_bytes(16, 16, 1024, 1, 0)
    pts = list(range(30, 38))
    with B.Ring(rb * room + rb // 2 // 64 * 64, 1 << 22) as ring:
        ring.set_policy(B.POLICY_DROP_NEWEST)
        s = torch.cuda.current_stream()
        for step in range(3):
            ring.observe_batch(pts, ts, reqs, step_id=step, stream=s.cuda_stream)
            s.synchronize()
            ring.drain(B.DRAIN_FLUSH)
            views = ring.poll_host()
            assert [v.seq for v in views] == [8 * step + i for i in range(room)]
            for i, v in enumerate(views):
                ref = orc.build_record(ts[i].cpu(), reqs, seq=v.seq, step_id=step, point_id=pts[i], out_dtype=1)
                assert np.array_equal(v.bytes(), ref)
            ring.release_host(views[-1].seq)
        st = ring.get_stats()
        assert (st.captured_records, st.dropped_records, st.launched_records) == (3 * room, 3 * (8 - room), 24)
        assert st.dropped_bytes == 3 * (8 - room) * rb and st.dropped_rows == 3 * (8 - room) * 16
        assert [ring.get_point_drops(p) for p in pts] == [0] * room + [3] * (8 - room)


def test_block_policy_splits_a_batch_that_exceeds_the_ring(B, run_gpu):
    """Device ring of 2 records, batches of 8 under the completeness policy: the library issues
    the batch in pieces and waits for the drain in between; nothing is lost."""
    wl = configs.config1_tiny(device=DEV)
    got = run_gpu(wl, device_ring_bytes=4352, host_ring_bytes=8192, poison=0x5A, batch=128)
    assert np.array_equal(got.stream, run_workload(wl).stream())
    assert got.stats.dev_ring_high_water <= 4352


# ------------------------------------------------------------------ whole workloads, batched
def test_config1_batched_equals_oracle_stream(run_gpu):
    wl = configs.config1_tiny(device=DEV)
    got = run_gpu(wl, poison=0xA5, batch=128)
    assert np.array_equal(got.stream, run_workload(wl).stream())
    got = run_gpu(wl, device_ring_bytes=8192, host_ring_bytes=16384, poison=0xA5, batch=3)
    assert np.array_equal(got.stream, run_workload(wl).stream())


def test_config2_batched_with_summaries(run_gpu):
    wl = configs.config2_decode8b(device=DEV, n_points=6, n_steps=5,
                                  device_ring_bytes=4 << 20, host_ring_bytes=8 << 20)
    got = run_gpu(wl, poison=0xA5, batch=128)
    assert got.stats.captured_records == 30
    compare_streams(got.stream, run_workload(wl).stream())


def test_config3_batched_fp8(run_gpu):
    wl = configs.config3_prefill(device=DEV, n_reqs=5, len_lo=30, len_hi=300, n_steps=2, hidden=4096,
                                 inter=14336, n_resid=3, n_mlp=2, device_ring_bytes=64 << 20,
                                 host_ring_bytes=64 << 20)
    got = run_gpu(wl, poison=0xA5, batch=128)
    ref = run_workload(wl)
    assert ref.stats.dropped_records == 0
    assert np.array_equal(got.stream, ref.stream())


def test_config4_batched_paged_kv(run_gpu):
    wl = configs.config4_paged_kv(device=DEV, n_layers_cap=2, n_blocks=1024, n_reqs=12, ctx_lo=20,
                                  ctx_hi=700, reqs_per_step=4, n_steps=3,
                                  device_ring_bytes=16 << 20, host_ring_bytes=32 << 20)
    got = run_gpu(wl, poison=0xA5, batch=128)
    assert np.array_equal(got.stream, run_workload(wl).stream())
    assert got.stats.captured_records == 2 * 2 * 3


@pytest.mark.parametrize("k", [1, 2])
def test_config5_batched_lockstep_drops_and_sampling(run_gpu, k):
    # device ring holds 3 records of 4,198,464 bytes; drain only every 2nd step; 5 points per batch
    wl = configs.config5_saturation(device=DEV, n_points=5, n_steps=8, sample_k=k,
                                    device_ring_bytes=13 << 20, host_ring_bytes=64 << 20)
    got = run_gpu(wl, drain_every=2, batch=128)
    ref = run_workload(wl, drain_every=2)
    assert np.array_equal(got.stream, ref.stream())
    a, b = got.stats, ref.stats
    assert (a.dropped_records, a.dropped_rows, a.dropped_bytes) == (b.dropped_records, b.dropped_rows, b.dropped_bytes)
    assert (a.sampled_out_calls, a.sampled_out_rows) == (b.sampled_out_calls, b.sampled_out_rows)
    assert a.captured_records == b.captured_records and a.launched_records == ref.next_seq
    if k == 1:
        assert b.dropped_records > 0


# ------------------------------------------------------------------ batched launches inside replayed steps
def _check_stats(run, ref):
    for k in ("observed_calls", "captured_records", "captured_rows", "captured_bytes", "dropped_records",
              "dropped_rows", "dropped_bytes", "sampled_out_calls", "sampled_out_rows"):
        assert getattr(run.stats, k) == getattr(ref.stats, k), k


@pytest.mark.parametrize("batch,extra", [(128, 0), (128, 2), (2, 3)])
def test_replayed_step_with_batched_launches(B, batch, extra):
    """11 hooks per step captured as 4 launches (5 + 3 + 2 + 1 records), or, with at most two per
    launch, as 7: an odd and an even number of launches per step, with ordinary observes between
    replays, exercise the hand-over of head and tail between the two copies of the control words."""
    from oracle import replay as oreplay
    from paper_2605_11093_amd import replay as G
    wl = configs.replayed_batches(n_steps=5, eager_extra_every=extra)
    ref = oreplay.run_workload(wl)
    run = G.run_workload_graph(wl, batch=batch)
    compare_streams(run.stream, ref.stream())
    _check_stats(run, ref)
    assert run.stats.bad_rows == 0


def test_replayed_step_with_a_long_batch_of_long_rows(B):
    """A replayed step whose last group (3 tensors, ~2,000 ragged rows of 4 KiB each, fp8) is one launch with
    more work than fits the GPU at once; the row counts change from replay to replay.  Then the same
    under best effort with a device ring of about one and a half steps, drained every second step."""
    from oracle import replay as oreplay
    from oracle.stream import POLICY_DROP_NEWEST
    from paper_2605_11093_amd import replay as G
    wl = configs.replayed_batches(n_steps=4, long_rows=3, device_ring_bytes=64 << 20, host_ring_bytes=128 << 20)
    ref = oreplay.run_workload(wl)
    run = G.run_workload_graph(wl, batch=128)
    compare_streams(run.stream, ref.stream())
    _check_stats(run, ref)
    wl = configs.replayed_batches(n_steps=4, long_rows=3, policy_mode=POLICY_DROP_NEWEST, device_ring_bytes=19 << 20,
                                  host_ring_bytes=128 << 20)
    ref = oreplay.run_workload(wl, drain_every=2)
    assert ref.stats.dropped_records > 0 and ref.stats.captured_records > 0
    run = G.run_workload_graph(wl, drain_every=2, batch=128)
    compare_streams(run.stream, ref.stream())
    _check_stats(run, ref)


def test_replayed_batches_sampled_out_and_drop_newest(B):
    from oracle import replay as oreplay
    from oracle.stream import POLICY_DROP_NEWEST
    from paper_2605_11093_amd import replay as G
    wl = configs.replayed_batches(n_steps=6, sample_k=2, eager_extra_every=2)
    ref = oreplay.run_workload(wl)
    run = G.run_workload_graph(wl, batch=128)
    compare_streams(run.stream, ref.stream())
    _check_stats(run, ref)
    # device ring holds about one and a half steps (a step is ~0.9 MB); drains every second step
    wl = configs.replayed_batches(n_steps=6, policy_mode=POLICY_DROP_NEWEST, device_ring_bytes=1344 << 10)
    ref = oreplay.run_workload(wl, drain_every=2)
    assert ref.stats.dropped_records > 0 and ref.stats.captured_records > 0
    run = G.run_workload_graph(wl, drain_every=2, batch=128)
    compare_streams(run.stream, ref.stream())
    _check_stats(run, ref)
