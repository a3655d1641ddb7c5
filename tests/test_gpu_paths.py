"""Every copy path of the capture kernels, with records wrapping the device ring at
varying offsets, and the device-side bounds handling.  Streams are compared with
the oracle's (bit-exact except the fp32 summaries, see _util)."""
import numpy as np
import pytest
import torch

import oracle as orc
from oracle.decode import decode_record
from oracle.stream import OracleRing, POLICY_BLOCK
from workloads import configs, prng
from _util import compare_record, compare_streams

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


def _stream_through_small_ring(B, make_call_args, n_obs, rec_bytes, paged=None):
    """n_obs observes through a device ring of ~2.3 records (so that records wrap at
    many different offsets) under the completeness policy; returns (gpu stream, oracle stream)."""
    dev_cap = max(4096, (int(rec_bytes * 2.3) // 64 + 1) * 64)
    host_cap = max(4096, (int(rec_bytes * 3.1) // 64 + 1) * 64)
    ref = OracleRing(dev_cap, host_cap, POLICY_BLOCK)
    got = []
    with B.Ring(dev_cap, host_cap, block_timeout_ms=1, max_reqs_per_observe=4096) as ring:
        ring.debug_fill_rings(0xA5)
        s = torch.cuda.current_stream()

        def consume():
            vs = ring.poll_host()
            for v in vs:
                got.append(v.bytes())
            if vs:
                ring.release_host(vs[-1].seq)
            seqs = ref.polled_seqs()
            if seqs:
                ref.release(seqs[-1])

        for i in range(n_obs):
            tensor, reqs, kw, okw = make_call_args(i)
            while True:
                if paged is None:
                    rc = ring.observe_tensor(i % 5, tensor, reqs, step_id=i, stream=s.cuda_stream,
                                             allow=(B.ERR_AGAIN,), **kw)
                else:
                    rc = ring.observe_paged(i % 5, tensor, paged.block_table, reqs, block_size=paged.block_size,
                                            n_heads=paged.n_heads, head_dim=paged.head_dim,
                                            heads_sel=paged.heads_sel, step_id=i, stream=s.cuda_stream,
                                            allow=(B.ERR_AGAIN,), **kw)
                if rc != B.ERR_AGAIN:
                    break
                s.synchronize()
                ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
                consume()
            cpu_paged = None if paged is None else configs.PagedSpec(paged.block_size, paged.n_heads, paged.head_dim,
                                                                     paged.heads_sel, paged.block_table.cpu())
            while True:
                rc = ref.observe(tensor.cpu(), reqs, point_id=i % 5, step_id=i, paged=cpu_paged, **okw)
                if rc != -5:
                    break
                ref.drain()
                seqs = ref.polled_seqs()
                if seqs:
                    ref.release(seqs[-1])
            assert rc == 0
        s.synchronize()
        for _ in range(1000):
            ring.drain(B.DRAIN_FLUSH, allow=(B.ERR_AGAIN,))
            consume()
            if ring.last_drain_status == B.OK:
                break
        st = ring.get_stats()
        assert st.dropped_records == 0 and st.bad_rows == 0
    while ref.drained < ref.appended:
        ref.drain()
        seqs = ref.polled_seqs()
        if seqs:
            ref.release(seqs[-1])
    return np.concatenate(got), ref.stream()


CASES = {
    # name: (T, E, dtype, reqs builder, out_dtype, summary_mask)
    "decode_lean_sum": (64, 4096, torch.bfloat16, "ones", 1, 5),
    "decode_lean_fp8": (256, 8192, torch.bfloat16, "ones", 4, 0),
    "decode_generic_fp16src": (64, 4096, torch.float16, "ones", 2, 7),
    "decode_generic_fp32src": (48, 1024, torch.float32, "ones", 3, 0),
    "long_rows_single_item": (300, 14336, torch.bfloat16, "ragged", 4, 0),
    "long_rows_multi_item": (40, 20480, torch.bfloat16, "ragged", 1, 0),
    "multi_row_items_512": (900, 4096, torch.bfloat16, "ragged", 4, 0),
    "multi_row_items_256": (900, 2048, torch.bfloat16, "ragged", 1, 0),
    "summ_wg_per_row_multipass": (60, 14336, torch.bfloat16, "ragged", 1, 7),
    "summ_wave_per_row_mid": (5000, 2048, torch.bfloat16, "ragged", 4, 5),
    "summ_wave_per_row_short": (700, 512, torch.bfloat16, "ragged", 2, 7),
    "short_rows_flat": (3000, 256, torch.bfloat16, "ragged", 1, 0),
    "elementwise_odd": (120, 1001, torch.bfloat16, "ragged", 4, 7),
    "summary_only_long": (2100, 8192, torch.bfloat16, "ragged", 0, 7),
    # few rows in all: the decode-shaped kernel with the host's row list
    "ragged_small_raw_sum": (220, 4096, torch.bfloat16, "ragged", 1, 5),
    "ragged_small_fp8": (220, 1024, torch.bfloat16, "ragged", 4, 0),
    "ragged_small_fp16_sum": (75, 8192, torch.bfloat16, "ragged", 2, 7),
    "ragged_small_summary_only": (1000, 256, torch.bfloat16, "ragged", 0, 3),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_path_through_a_wrapping_ring(B, name):
    T, E, dt, kind, out_dtype, sm = CASES[name]
    pool = [prng.randn_bf16(prng.sub_seed(31, len(name), k), T * E, DEV).view(T, E).to(dt) for k in range(2)]
    if kind == "ones":
        reqs = np.array([(i, i, 0, 1, 1) for i in range(T)], dtype=np.uint32)
    else:
        n = 7
        per = T // n
        reqs = np.array([(100 + i, i * per, i % 3, max(1, (per - 3) // (1 + i % 2)), 1 + i % 2) for i in range(n)],
                        dtype=np.uint32)
    rows = int(reqs[:, 3].sum())
    rec = orc.record_bytes(len(reqs), rows, E, out_dtype, sm)

    def args(i):
        kw = dict(out_dtype=out_dtype, summary_mask=sm)
        return pool[i % 2], reqs, kw, kw

    got, ref = _stream_through_small_ring(B, args, 9, rec)
    compare_streams(got, ref)


def test_paged_path_through_a_wrapping_ring(B):
    NB, BS, NH, HD = 256, 16, 8, 128
    cache = prng.randn_bf16(prng.sub_seed(32, 1), NB * BS * NH * HD, DEV).view(NB, BS, NH, HD)
    table = torch.from_numpy(prng.permutation(5, NB).astype(np.int32).reshape(8, 32)).to(DEV)
    spec = configs.PagedSpec(BS, NH, HD, [1, 5], table)
    reqs = np.array([(1, 0, 0, 500, 1), (2, 3, 7, 300, 1), (3, 7, 0, 170, 3)], dtype=np.uint32)
    rec = orc.record_bytes(3, 970, 256, 1, 0)

    def args(i):
        kw = dict(out_dtype=1 if i % 2 else 4, summary_mask=0)
        return cache, reqs, kw, kw

    got, ref = _stream_through_small_ring(B, args, 8, rec, paged=spec)
    compare_streams(got, ref)


def test_four_thousand_requests_with_mask_and_index(B):
    n = 4096
    t = prng.randn_bf16(prng.sub_seed(33, 1), 6000 * 128, DEV).view(6000, 128)
    reqs = np.array([(i, i, 0, 1 + (i % 3 == 0), 1) for i in range(n)], dtype=np.uint32)
    mask = (np.arange(n) % 5 != 2).astype(np.uint8)
    listed = int(reqs[:, 3].sum())
    idx = ((np.arange(listed) * 7919) % 6000).astype(np.int32)
    with B.Ring(1 << 23, 1 << 23, max_reqs_per_observe=4096) as ring:
        s = torch.cuda.current_stream()
        km = torch.from_numpy(mask).to(DEV)
        ri = torch.from_numpy(idx).to(DEV)
        ring.observe_tensor(0, t, reqs, step_id=0, stream=s.cuda_stream, keep_mask=km, summary_mask=7)
        ring.observe_tensor(1, t, reqs, step_id=0, stream=s.cuda_stream, keep_mask=km, row_index=ri, out_dtype=4)
        ring.observe_tensor(2, t, reqs, step_id=0, stream=s.cuda_stream, row_index=ri)
        ring.drain(B.DRAIN_FLUSH)
        v = ring.poll_host()
        assert len(v) == 3
        tc = t.cpu()
        compare_record(v[0].bytes(), orc.build_record(tc, reqs, seq=0, step_id=0, point_id=0, out_dtype=1,
                                                      summary_mask=7, keep_mask=mask))
        compare_record(v[1].bytes(), orc.build_record(tc, reqs, seq=1, step_id=0, point_id=1, out_dtype=4,
                                                      keep_mask=mask, row_index=idx))
        compare_record(v[2].bytes(), orc.build_record(tc, reqs, seq=2, step_id=0, point_id=2, out_dtype=1,
                                                      row_index=idx))


def test_out_of_range_device_indices_give_zero_rows_and_are_counted(B):
    t = prng.randn_bf16(prng.sub_seed(34, 1), 50 * 512, DEV).view(50, 512)
    reqs = np.array([(i, 0, 0, 1, 1) for i in range(6)], dtype=np.uint32)
    idx = np.array([3, 50, 7, -1, 49, 1 << 20], dtype=np.int32)          # three of them leave the tensor
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream()
        ri = torch.from_numpy(idx).to(DEV)
        ring.observe_tensor(0, t, reqs, step_id=0, stream=s.cuda_stream, row_index=ri, summary_mask=5)
        ring.drain(B.DRAIN_FLUSH)
        r = decode_record(ring.poll_host()[0].bytes())
        bits = t.cpu().view(torch.int16).numpy().astype(np.uint16)
        for g, src in enumerate(idx):
            if 0 <= src < 50:
                assert (r.payload[g] == bits[src]).all()
            else:
                assert not r.payload[g].any() and r.summaries[1][g] == 0 and r.summaries[4][g] == 0
        assert ring.get_stats().bad_rows == 3
    # the general kernel's summary pass (an fp32 source keeps the launch off the decode-shaped kernel),
    # a workgroup per row (E = 8200) and a wavefront per row (E = 96)
    for E in (8200, 96):
        t32 = prng.randn_bf16(prng.sub_seed(34, 3, E), 50 * E, DEV).view(50, E).float()
        with B.Ring(1 << 22, 1 << 22) as ring:
            s = torch.cuda.current_stream()
            ri = torch.from_numpy(idx).to(DEV)
            ring.observe_tensor(0, t32, reqs, step_id=0, stream=s.cuda_stream, row_index=ri, summary_mask=7)
            ring.drain(B.DRAIN_FLUSH)
            r = decode_record(ring.poll_host()[0].bytes())
            src32 = t32.cpu().numpy()
            for g, src in enumerate(idx):
                if 0 <= src < 50:
                    assert (r.payload[g] == src32[src]).all()
                    assert r.summaries[4][g] == np.abs(src32[src]).max()
                    assert abs(r.summaries[1][g] - np.sqrt((src32[src].astype(np.float64) ** 2).sum())) <= 1e-3 * r.summaries[1][g]
                else:
                    assert not r.payload[g].any() and r.summaries[1][g] == 0 and r.summaries[4][g] == 0
            assert ring.get_stats().bad_rows == 3, E
    # a block-table entry beyond the cache
    NB, BS, NH, HD = 8, 16, 2, 128
    cache = prng.randn_bf16(prng.sub_seed(34, 2), NB * BS * NH * HD, DEV).view(NB, BS, NH, HD)
    table = torch.tensor([[0, 9, 2, 3]], dtype=torch.int32, device=DEV)    # 9 >= NB
    with B.Ring(1 << 20, 1 << 20) as ring:
        s = torch.cuda.current_stream()
        ring.observe_paged(0, cache, table, np.array([(1, 0, 0, 40, 1)], np.uint32), block_size=BS, n_heads=NH,
                           head_dim=HD, heads_sel=[1], step_id=0, stream=s.cuda_stream)
        ring.drain(B.DRAIN_FLUSH)
        r = decode_record(ring.poll_host()[0].bytes())
        bits = cache.cpu().view(torch.int16).numpy().astype(np.uint16)
        for tkn in range(40):
            blk = [0, 9, 2, 3][tkn // BS]
            if blk < NB:
                assert (r.payload[tkn] == bits[blk, tkn % BS, 1]).all()
            else:
                assert not r.payload[tkn].any()
        assert ring.get_stats().bad_rows == 16


MASKED_DECODE = {
    # name: (n_reqs, E, out_dtype, summary_mask, mask kind, row placement)
    "c2_shape": (64, 4096, 1, 5, "mod4", "consecutive"),
    "fp8_1000_reqs": (1000, 512, 4, 0, "random", "consecutive"),
    "fp16_permuted_rows": (300, 1024, 2, 7, "random", "permuted"),
    "all_out": (70, 256, 1, 7, "none", "consecutive"),
    "all_in_indexed": (129, 8192, 1, 1, "all", "indexed"),
    "summary_only": (257, 2048, 0, 7, "random", "consecutive"),
    "one_request": (1, 4096, 1, 5, "all", "consecutive"),
    "one_request_out": (1, 4096, 4, 0, "none", "consecutive"),
}


@pytest.mark.parametrize("name", sorted(MASKED_DECODE))
def test_keep_vector_on_decode_shapes_through_a_wrapping_ring(B, name):
    """One row per request with a keep vector (the best-effort path of a decode step)."""
    n, E, out_dtype, sm, mkind, place = MASKED_DECODE[name]
    T = n + 3
    pool = [prng.randn_bf16(prng.sub_seed(34, len(name), k), T * E, DEV).view(T, E) for k in range(2)]
    if place == "permuted":
        rows = prng.permutation(prng.sub_seed(34, 7), T)[:n]
    else:
        rows = np.arange(n) + 2
    reqs = np.array([(9000 + i, int(rows[i]), 0, 1, 1) for i in range(n)], dtype=np.uint32)
    idx = None
    if place == "indexed":
        idx = ((np.arange(n) * 31) % T).astype(np.int32)
    masks = []
    for k in range(3):
        if mkind == "mod4":
            m = ((np.arange(n) + k) % 4 != 1)
        elif mkind == "random":
            m = prng.randint(prng.sub_seed(34, 8, k), n, 0, 2) > 0
        elif mkind == "none":
            m = np.zeros(n, bool)
        else:
            m = np.ones(n, bool)
        masks.append(m.astype(np.uint8))
    dev_masks = [torch.from_numpy(m).to(DEV) for m in masks]
    dev_idx = None if idx is None else torch.from_numpy(idx).to(DEV)
    rec = orc.record_bytes(n, n, E, out_dtype, sm)

    def args(i):
        kw = dict(out_dtype=out_dtype, summary_mask=sm, keep_mask=dev_masks[i % 3])
        okw = dict(out_dtype=out_dtype, summary_mask=sm, keep_mask=masks[i % 3])
        if idx is not None:
            kw["row_index"] = dev_idx
            okw["row_index"] = idx
        return pool[i % 2], reqs, kw, okw

    got, ref = _stream_through_small_ring(B, args, 9, rec)
    compare_streams(got, ref)
    for rbytes in (decode_record(got[:0 + int.from_bytes(got[48:56].tobytes(), "little")]),):
        assert rbytes.flags & 2


@pytest.mark.parametrize("n,rows_each,masked", [(1024, 1, True), (1025, 1, True), (512, 2, False), (513, 2, False),
                                                 (341, 3, False), (342, 3, False)])
def test_kernel_choice_boundaries(B, n, rows_each, masked):
    """Just inside and just outside what the decode-shaped kernel takes (1024 requests with
    a keep vector; 1024 listed rows without): both sides must give the oracle's record."""
    E = 256
    T = n * rows_each + 5
    t = prng.randn_bf16(prng.sub_seed(35, n, rows_each), T * E, DEV).view(T, E)
    reqs = np.array([(i, 2 + i * rows_each, 0, rows_each, 1) for i in range(n)], dtype=np.uint32)
    mask = (prng.randint(prng.sub_seed(35, 9, n), n, 0, 3) > 0).astype(np.uint8) if masked else None
    with B.Ring(8 << 20, 8 << 20, max_reqs_per_observe=2048) as ring:
        s = torch.cuda.current_stream()
        km = None if mask is None else torch.from_numpy(mask).to(DEV)
        ring.observe_tensor(3, t, reqs, step_id=11, stream=s.cuda_stream, keep_mask=km, summary_mask=5)
        ring.observe_tensor(4, t, reqs, step_id=11, stream=s.cuda_stream, keep_mask=km, out_dtype=4)
        ring.drain(B.DRAIN_FLUSH)
        v = ring.poll_host()
        tc = t.cpu()
        compare_record(v[0].bytes(), orc.build_record(tc, reqs, seq=0, step_id=11, point_id=3, out_dtype=1,
                                                      summary_mask=5, keep_mask=mask))
        compare_record(v[1].bytes(), orc.build_record(tc, reqs, seq=1, step_id=11, point_id=4, out_dtype=4,
                                                      keep_mask=mask))


PAGED_RANGES = {
    # name: (cache dtype, out_dtype, heads, requests (id, table row, first token, tokens, step), keep vector?)
    "mid_block_starts": (torch.bfloat16, 1, [1, 5], [(1, 0, 5, 300, 1), (2, 3, 0, 16, 1), (3, 7, 15, 2, 1),
                                                     (4, 2, 31, 97, 1)], False),
    "fp8_with_empty_requests": (torch.bfloat16, 4, [0, 7], [(1, 1, 0, 0, 1), (2, 2, 3, 250, 1), (3, 3, 9, 0, 1),
                                                            (4, 4, 100, 1, 1), (5, 5, 0, 0, 1)], False),
    "fp16_keep_vector": (torch.bfloat16, 2, [2], [(10 + i, i % 8, 3 * i, 40 + 7 * i, 1) for i in range(9)], True),
    "fp32_cache": (torch.float32, 3, [3, 4], [(1, 6, 2, 77, 1), (2, 5, 16, 48, 1)], False),
    "seventy_requests": (torch.bfloat16, 1, [6], [(i, i % 8, (5 * i) % 64, 1 + (11 * i) % 50, 1) for i in range(70)], True),
}


@pytest.mark.parametrize("name", sorted(PAGED_RANGES))
def test_paged_token_ranges_through_a_wrapping_ring(B, name):
    """Contiguous token ranges out of a paged cache: ranges that start and end inside
    blocks, empty requests, keep vectors, an fp32 cache."""
    dt, out_dtype, heads, req_list, masked = PAGED_RANGES[name]
    NB, BS, NH, HD = 256, 16, 8, 128 if dt != torch.float32 else 64
    cache = prng.randn_bf16(prng.sub_seed(36, len(name)), NB * BS * NH * HD, DEV).view(NB, BS, NH, HD).to(dt)
    table = torch.from_numpy(prng.permutation(prng.sub_seed(36, 2), NB).astype(np.int32).reshape(8, 32)).to(DEV)
    spec = configs.PagedSpec(BS, NH, HD, heads, table)
    reqs = np.array(req_list, dtype=np.uint32)
    n = len(req_list)
    rows = int(reqs[:, 3].sum())
    rec = orc.record_bytes(n, rows, len(heads) * HD, out_dtype, 0)
    masks = [(prng.randint(prng.sub_seed(36, 3, k), n, 0, 2) > 0).astype(np.uint8) for k in range(3)]
    dev_masks = [torch.from_numpy(m).to(DEV) for m in masks]

    def args(i):
        kw, okw = dict(out_dtype=out_dtype, summary_mask=0), dict(out_dtype=out_dtype, summary_mask=0)
        if masked:
            kw["keep_mask"], okw["keep_mask"] = dev_masks[i % 3], masks[i % 3]
        return cache, reqs, kw, okw

    got, ref = _stream_through_small_ring(B, args, 8, rec, paged=spec)
    compare_streams(got, ref)


@pytest.mark.parametrize("out_dtype,sm,masked", [(2, 7, False), (2, 0, True), (0, 5, True), (2, 3, True)])
def test_fp16_source_on_decode_shapes(B, out_dtype, sm, masked):
    n, E = 130, 2048
    pool = [prng.randn_bf16(prng.sub_seed(37, k), (n + 1) * E, DEV).view(n + 1, E).to(torch.float16) for k in range(2)]
    reqs = np.array([(i, i + 1, 0, 1, 1) for i in range(n)], dtype=np.uint32)
    masks = [(prng.randint(prng.sub_seed(37, 5, k), n, 0, 3) > 0).astype(np.uint8) for k in range(2)]
    dev_masks = [torch.from_numpy(m).to(DEV) for m in masks]
    rec = orc.record_bytes(n, n, E, out_dtype, sm)

    def args(i):
        kw, okw = dict(out_dtype=out_dtype, summary_mask=sm), dict(out_dtype=out_dtype, summary_mask=sm)
        if masked:
            kw["keep_mask"], okw["keep_mask"] = dev_masks[i % 2], masks[i % 2]
        return pool[i % 2], reqs, kw, okw

    got, ref = _stream_through_small_ring(B, args, 7, rec)
    compare_streams(got, ref)
