"""Parity of the HIP path with the CPU oracle, through the C ABI, on sizes the
oracle finishes in seconds: all five workload shapes scaled down so that they
still span several tiles and ragged tails, plus the method's edge cases."""
import hashlib
import json
import os

import numpy as np
import pytest
import torch

import oracle as orc
from oracle.replay import run_workload
from oracle.stream import OracleRing
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


def _one(B, tensor, reqs, *, out_dtype=None, summary_mask=0, keep_mask=None, row_index=None,
         paged=None, ring_bytes=1 << 22, poison=0xA5):
    """One observe on a fresh, poisoned ring -> (gpu record bytes, oracle record bytes)."""
    reqs = np.asarray(reqs, dtype=np.uint32).reshape(-1, 5)
    with B.Ring(ring_bytes, ring_bytes) as ring:
        ring.debug_fill_rings(poison)
        s = torch.cuda.current_stream()
        km = None if keep_mask is None else torch.tensor(keep_mask, dtype=torch.uint8, device=DEV)
        ri = None if row_index is None else torch.tensor(row_index, dtype=torch.int32, device=DEV)
        src_dt = {torch.bfloat16: 1, torch.float16: 2, torch.float32: 3}[tensor.dtype]
        od = src_dt if out_dtype is None else out_dtype
        before = tensor.clone()
        if paged is None:
            ring.observe_tensor(3, tensor, reqs, step_id=11, stream=s.cuda_stream, out_dtype=od,
                                summary_mask=summary_mask, keep_mask=km, row_index=ri)
        else:
            ring.observe_paged(3, tensor, paged.block_table, reqs, block_size=paged.block_size,
                               n_heads=paged.n_heads, head_dim=paged.head_dim, heads_sel=paged.heads_sel,
                               step_id=11, stream=s.cuda_stream, out_dtype=od,
                               summary_mask=summary_mask, keep_mask=km)
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert len(views) == 1 and views[0].seq == 0
        got = views[0].bytes()
        s.synchronize()
        assert torch.equal(before.view(torch.uint8), tensor.view(torch.uint8)), "observed tensor was modified"
    cpu_paged = None
    if paged is not None:
        cpu_paged = configs.PagedSpec(paged.block_size, paged.n_heads, paged.head_dim, paged.heads_sel,
                                      paged.block_table.cpu())
    ref = orc.build_record(tensor.cpu(), reqs, seq=0, step_id=11, point_id=3, out_dtype=od,
                           summary_mask=summary_mask, keep_mask=keep_mask, row_index=row_index,
                           paged=cpu_paged)
    return got, ref


# ------------------------------------------------------------------ config 1
def test_config1_stream_is_oracle_exact_and_matches_golden(run_gpu):
    wl = configs.config1_tiny(device=DEV)
    got = run_gpu(wl, poison=0xA5)
    ref = run_workload(wl).stream()
    assert np.array_equal(got.stream, ref)
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "config1_stream.json")))
    assert hashlib.sha256(got.stream.tobytes()).hexdigest() == gold["sha256"]
    st = got.stats
    assert (st.captured_records, st.captured_rows, st.captured_bytes) == (128, 512, 278528)
    assert st.dropped_records == 0 and st.drained_bytes == 278528 and st.released_bytes == 278528


@pytest.mark.parametrize("dev,host", [(8192, 16384), (4352, 4096), (4096, 8192)])
def test_config1_wraps_many_times_with_tiny_rings(run_gpu, dev, host):
    wl = configs.config1_tiny(device=DEV)
    got = run_gpu(wl, device_ring_bytes=dev, host_ring_bytes=host, poison=0x5A)
    assert np.array_equal(got.stream, run_workload(wl).stream())
    assert got.stats.dev_ring_high_water <= dev and got.stats.host_ring_high_water <= host


@pytest.mark.parametrize("flags_name", ["DRAIN_KERNEL", "BG_THREAD"])
def test_config1_other_drain_modes(B, run_gpu, flags_name):
    wl = configs.config1_tiny(device=DEV)
    got = run_gpu(wl, device_ring_bytes=8192, host_ring_bytes=16384, flags=getattr(B, flags_name), poison=0xA5)
    assert np.array_equal(got.stream, run_workload(wl).stream())


# ------------------------------------------------------------------ configs 2-5, scaled
def test_config2_decode_with_summaries(run_gpu):
    wl = configs.config2_decode8b(device=DEV, n_points=3, n_steps=5,
                                  device_ring_bytes=2 << 20, host_ring_bytes=3 << 20)
    got = run_gpu(wl, poison=0xA5)
    ref = run_workload(wl)
    assert got.stats.captured_records == 15 and got.stats.captured_bytes == 15 * 525888
    compare_streams(got.stream, ref.stream())


def test_config3_ragged_prefill_fp8(run_gpu):
    wl = configs.config3_prefill(device=DEV, n_reqs=5, len_lo=30, len_hi=300, n_steps=2, hidden=4096,
                                 inter=14336, n_resid=2, n_mlp=1, device_ring_bytes=64 << 20,
                                 host_ring_bytes=64 << 20)
    got = run_gpu(wl, poison=0xA5)
    ref = run_workload(wl)
    assert ref.stats.dropped_records == 0
    assert np.array_equal(got.stream, ref.stream())


def test_config4_paged_kv(run_gpu):
    wl = configs.config4_paged_kv(device=DEV, n_layers_cap=2, n_blocks=1024, n_reqs=12, ctx_lo=20,
                                  ctx_hi=700, reqs_per_step=4, n_steps=3,
                                  device_ring_bytes=16 << 20, host_ring_bytes=32 << 20)
    got = run_gpu(wl, poison=0xA5)
    ref = run_workload(wl)
    assert np.array_equal(got.stream, ref.stream())
    assert got.stats.captured_records == 2 * 2 * 3


@pytest.mark.parametrize("k", [1, 2, 4])
def test_config5_saturation_lockstep_drops_and_sampling(run_gpu, k):
    # device ring holds 3 records of 4,198,464 bytes; drain only every 2nd step
    wl = configs.config5_saturation(device=DEV, n_points=5, n_steps=8, sample_k=k,
                                    device_ring_bytes=13 << 20, host_ring_bytes=64 << 20)
    got = run_gpu(wl, drain_every=2)
    ref = run_workload(wl, drain_every=2)
    assert np.array_equal(got.stream, ref.stream())
    a, b = got.stats, ref.stats
    assert (a.dropped_records, a.dropped_rows, a.dropped_bytes) == (b.dropped_records, b.dropped_rows, b.dropped_bytes)
    assert (a.sampled_out_calls, a.sampled_out_rows) == (b.sampled_out_calls, b.sampled_out_rows)
    assert a.captured_records == b.captured_records and a.launched_records == ref.next_seq
    if k == 1:
        assert b.dropped_records > 0


# ------------------------------------------------------------------ gathers: shapes and alignment
@pytest.mark.parametrize("E", [1, 3, 8, 250, 257, 264, 2048, 2056, 5120])
@pytest.mark.parametrize("offset_elems", [0, 1, 8])
def test_dense_gather_any_width_and_alignment(B, E, offset_elems):
    T, pitch = 37, E + 24
    buf = prng.randn_bf16(prng.sub_seed(99, E), T * pitch + 16, DEV)
    t = buf[offset_elems: offset_elems + T * pitch].view(T, pitch)[:, :E]
    reqs = [(1, 0, 2, 3, 1), (2, 10, 0, 6, 4), (3, 36, 0, 1, 1), (4, 5, 0, 0, 1)]
    got, ref = _one(B, t, reqs)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("src", [torch.float16, torch.float32])
@pytest.mark.parametrize("E", [6, 512])
def test_raw_copy_of_other_source_dtypes(B, src, E):
    t = prng.randn_bf16(5, 40 * E, DEV).view(40, E).to(src)
    got, ref = _one(B, t, [(1, 3, 1, 9, 2), (2, 30, 0, 10, 1)], summary_mask=7)
    compare_record(got, ref)


def test_keep_mask_and_row_index(B):
    t = prng.randn_bf16(6, 300 * 512, DEV).view(300, 512)
    reqs = [(10 + i, 20 * i, 0, 3 + i, 2) for i in range(9)]
    mask = [1, 0, 1, 1, 0, 0, 1, 0, 1]
    got, ref = _one(B, t, reqs, keep_mask=mask, summary_mask=5)
    compare_record(got, ref)
    n = sum(r[3] for r in reqs)
    idx = (np.arange(n) * 37 + 11) % 300
    got, ref = _one(B, t, reqs, row_index=idx)
    assert np.array_equal(got, ref)
    got, ref = _one(B, t, reqs, row_index=idx, keep_mask=mask, out_dtype=DT_FP8)
    assert np.array_equal(got, ref)
    got, ref = _one(B, t, reqs, keep_mask=[0] * 9)
    assert np.array_equal(got, ref) and got.size == 64 + 192


def test_same_launch_two_masks_gives_two_exact_records(B):
    """The keep/drop vector changes data, not topology: it is read when the kernel runs."""
    t = prng.randn_bf16(8, 64 * 256, DEV).view(64, 256)
    reqs = np.array([(i, i, 0, 1, 1) for i in range(64)], dtype=np.uint32)
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream()
        km = torch.ones(64, dtype=torch.uint8, device=DEV)
        m1 = (np.arange(64) % 3 != 0).astype(np.uint8)
        km.copy_(torch.from_numpy(m1))
        ring.observe_tensor(0, t, reqs, step_id=0, stream=s.cuda_stream, keep_mask=km)
        m2 = (np.arange(64) % 5 == 0).astype(np.uint8)
        km.copy_(torch.from_numpy(m2), non_blocking=False)
        ring.observe_tensor(0, t, reqs, step_id=1, stream=s.cuda_stream, keep_mask=km)
        ring.drain(B.DRAIN_FLUSH)
        v = ring.poll_host()
        assert len(v) == 2
        for view, m, step in zip(v, (m1, m2), (0, 1)):
            ref = orc.build_record(t.cpu(), reqs, seq=view.seq, step_id=step, point_id=0, out_dtype=1, keep_mask=m)
            assert np.array_equal(view.bytes(), ref)


def test_empty_and_degenerate_selections(B):
    t = prng.randn_bf16(7, 16 * 64, DEV).view(16, 64)
    got, ref = _one(B, t, np.zeros((0, 5), np.uint32))
    assert got.size == 64 and np.array_equal(got, ref)
    got, ref = _one(B, t, [(1, 0, 0, 0, 1), (2, 3, 0, 0, 1)], summary_mask=7)
    assert np.array_equal(got, ref)
    got, ref = _one(B, t, [(1, 5, 0, 4, 0)])           # tok_step 0: the same row four times
    assert np.array_equal(got, ref)
    got, ref = _one(B, t, [(1, 0, 0, 16, 1)], out_dtype=DT_NONE, summary_mask=0)   # nothing but a header
    assert np.array_equal(got, ref)


def test_many_requests_use_the_global_table_path(B):
    n = 1500                                            # above the LDS-cached table size
    t = prng.randn_bf16(9, 2000 * 64, DEV).view(2000, 64)
    reqs = [(i, i, 0, 1 + (i % 2), 1) for i in range(n)]
    with B.Ring(1 << 22, 1 << 22, max_reqs_per_observe=2048) as ring:
        s = torch.cuda.current_stream()
        mask = (np.arange(n) % 7 != 3).astype(np.uint8)
        km = torch.from_numpy(mask).to(DEV)
        ring.observe_tensor(1, t, np.array(reqs, np.uint32), step_id=2, stream=s.cuda_stream, keep_mask=km,
                            summary_mask=4)
        ring.drain(B.DRAIN_FLUSH)
        got = ring.poll_host()[0].bytes()
    ref = orc.build_record(t.cpu(), reqs, seq=0, step_id=2, point_id=1, out_dtype=1, summary_mask=4, keep_mask=mask)
    compare_record(got, ref)


# ------------------------------------------------------------------ downcasts and summaries
@pytest.mark.parametrize("out_dtype", [DT_FP8, DT_FP16])
@pytest.mark.parametrize("width", [256, 250])
def test_downcast_of_every_bf16_bit_pattern(B, out_dtype, width):
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    n = 65536 // 256 * width
    t = bits[:n].view(torch.bfloat16).view(-1, width).to(DEV)
    if width == 250:            # cover the patterns the narrower view cut off
        t = torch.cat([t, bits[-n:].view(torch.bfloat16).view(-1, width).to(DEV)])
    got, ref = _one(B, t, [(1, 0, 0, t.shape[0], 1)], out_dtype=out_dtype, ring_bytes=1 << 20)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("out_dtype", [DT_FP16, DT_FP8])
@pytest.mark.parametrize("shape", [(2048, 32), (16, 4096)])
def test_downcast_of_every_bf16_bit_pattern_general_kernel(B, out_dtype, shape):
    """The same exhaustive check through the general kernel's short-row and long-row paths
    (more than 1024 rows, or a keep vector with several rows per request, keep it off the
    decode-shaped kernel)."""
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    t = bits.view(torch.bfloat16).view(*shape).to(DEV)
    if shape[0] > 1024:
        got, ref = _one(B, t, [(1, 0, 0, shape[0], 1)], out_dtype=out_dtype, ring_bytes=1 << 20)
    else:
        got, ref = _one(B, t, [(1, 0, 0, 9, 1), (2, 9, 0, 7, 1)], out_dtype=out_dtype, keep_mask=[1, 1],
                        ring_bytes=1 << 20)
    assert np.array_equal(got, ref)


def test_summaries_closed_forms_and_non_finite(B):
    E = 4096
    x = torch.zeros(8, E, dtype=torch.bfloat16, device=DEV)
    x[0, :] = -1.5
    x[1, 17] = 3.0
    x[2, 0::2] = 1.0
    x[2, 1::2] = -1.0
    x[3] = prng.randn_bf16(3, E, DEV)
    x[4] = prng.randn_bf16(4, E, DEV)
    x[4, 100] = float("inf")
    x[5] = prng.randn_bf16(5, E, DEV)
    x[5, 7] = float("nan")
    x[6] = prng.randn_bf16(6, E, DEV) * 1e-3
    got, ref = _one(B, x, [(1, 0, 0, 8, 1)], out_dtype=DT_NONE, summary_mask=7)
    compare_record(got, ref)
    from oracle.decode import decode_record
    g = decode_record(got)
    assert g.summaries[1][0] == np.float32(1.5 * 64) and g.summaries[2][0] == -1.5 and g.summaries[4][0] == 1.5
    assert g.summaries[1][1] == 3.0 and g.summaries[4][1] == 3.0
    assert g.summaries[2][2] == 0.0 and g.summaries[1][2] == 64.0
    assert np.isnan(g.summaries[1][5]) and np.isnan(g.summaries[2][5])
    # true mean tolerance: 1e-3 |ref| + 1e-5 mean|x|
    v = x[3].double().cpu().numpy()
    assert abs(g.summaries[2][3] - v.mean()) <= 1e-3 * abs(v.mean()) + 1e-5 * np.abs(v).mean()


@pytest.mark.parametrize("rows_per_request", [1, 3])
def test_l2_limit_of_the_fp32_sum_of_squares(B, rows_per_request):
    """The documented limit of the L2 summary (include/dmi.h, dmi_transform_t): the kernels sum
    squares in fp32, the oracle in float64 rounded once.  Where the fp32 sum overflows although the
    norm itself is representable the stored L2 is +inf; where every square underflows it is 0.
    Mean and absmax are not affected, and just inside the limits the L2 is within tolerance.
    (Activations are nowhere near either end: |x| > 1.8e19 / sqrt(E) or |x| < 1e-22.)
    One row per request takes the decode-shaped kernel, three per request with a keep vector the
    general one."""
    from oracle.decode import decode_record
    E = 4096
    x = torch.zeros(6, E, dtype=torch.bfloat16, device=DEV)
    x[0, :] = 2.0 ** 70                      # sum of squares 2^152: beyond fp32; L2 = 2^76 is not
    x[1, 9] = torch.tensor([0x7F7F], dtype=torch.int16).view(torch.bfloat16)[0]     # largest finite bf16
    x[2, :] = 2.0 ** -80                     # squares underflow; L2 = 2^-74 is representable
    x[3, :] = 2.0 ** 57                      # sum of squares 2^126: still fine
    x[4, :] = -(2.0 ** -60)                  # squares 2^-120: still fine
    x[5] = prng.randn_bf16(77, E, DEV)
    if rows_per_request == 1:
        reqs, keep = [(i, i, 0, 1, 1) for i in range(6)], None
    else:
        reqs, keep = [(1, 0, 0, 3, 1), (2, 3, 0, 3, 1)], [1, 1]
    got, ref = _one(B, x, reqs, out_dtype=DT_NONE, summary_mask=7, keep_mask=keep)
    g, r = decode_record(got), decode_record(ref)
    assert np.array_equal(g.summaries[4], r.summaries[4])                                  # absmax exact
    assert g.summaries[4][1] == np.float32(3.3895313892515355e38)
    assert np.allclose(g.summaries[2], r.summaries[2], rtol=1e-3, atol=0)                  # means
    l2g, l2r = g.summaries[1], r.summaries[1]
    assert np.isfinite(l2r).all() and l2r[0] == np.float32(2.0 ** 76) and l2r[2] == np.float32(2.0 ** -74)
    assert np.isposinf(l2g[0]) and np.isposinf(l2g[1]) and l2g[2] == 0.0                   # the limit
    for i in (3, 4, 5):
        assert abs(float(l2g[i]) - float(l2r[i])) <= 1e-3 * float(l2r[i])


@pytest.mark.parametrize("E", [64, 257, 1024, 14336])
@pytest.mark.parametrize("out_dtype", [DT_BF16, DT_FP8])
def test_summaries_with_payload_across_row_lengths(B, E, out_dtype):
    t = prng.randn_bf16(prng.sub_seed(12, E), 21 * E, DEV).view(21, E)
    got, ref = _one(B, t, [(1, 0, 0, 11, 1), (2, 12, 1, 4, 2)], out_dtype=out_dtype, summary_mask=7)
    compare_record(got, ref)


# ------------------------------------------------------------------ paged gathers
@pytest.mark.parametrize("head_dim,heads_sel", [(128, [1, 5]), (64, [7, 0, 3]), (20, [2])])
def test_paged_gather_shapes(B, head_dim, heads_sel):
    NB, BS, NH = 64, 16, 8
    cache = prng.randn_bf16(prng.sub_seed(13, head_dim), NB * BS * NH * head_dim, DEV).view(NB, BS, NH, head_dim)
    table = torch.from_numpy(prng.permutation(3, NB).astype(np.int32).reshape(4, 16)).to(DEV)
    spec = configs.PagedSpec(BS, NH, head_dim, heads_sel, table)
    reqs = [(1, 2, 0, 200, 1), (2, 0, 5, 40, 3), (3, 3, 255, 1, 1)]
    got, ref = _one(B, cache, reqs, paged=spec)
    assert np.array_equal(got, ref)
    got, ref = _one(B, cache, reqs, paged=spec, keep_mask=[0, 1, 1], summary_mask=5, out_dtype=DT_FP8)
    compare_record(got, ref)
