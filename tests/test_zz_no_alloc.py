"""dmi_observe_into, the entry point that allocates nothing, against dmi_observe.

Both go through the C ABI.  The record dmi_observe_into writes into the caller's buffer must
be the record that dmi_observe produces for the same arguments (taken out of a ring by drain
and poll), byte for byte: copies, gathers, downcasts and layout are bit-exact work, and both
run the same kernels, so the fp32 summaries are compared bit-exactly too.  Two calls in a
row, the second with a smaller input, share the library's per-GPU scratch memory.  The oracle's
record is checked as well (to the summaries' tolerance)."""
import numpy as np
import pytest
import torch

import oracle as orc
from workloads import prng
from _util import compare_record

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
DT_BF16, DT_FP16, DT_FP8 = 1, 2, 4
POISON = 0xC3


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available()
    from paper_2605_11093_amd import binding
    binding.lib()
    return binding


def _via_ring(B, tensor, reqs, *, seq_before, step_id, rank_tag, out_dtype, summary_mask, keep_mask, row_index):
    """The existing entry point: dmi_observe into a ring -> drain -> poll.  `seq_before`
    throw-away observes come first so that the record of interest gets that sequence number."""
    s = torch.cuda.current_stream()
    with B.Ring(8 << 20, 8 << 20, rank_tag=rank_tag, max_reqs_per_observe=1024) as ring:
        one = np.array([[0, 0, 0, 1, 1]], dtype=np.uint32)
        for _ in range(seq_before):
            ring.observe_tensor(1, tensor, one, step_id=0, stream=s.cuda_stream)
        ring.observe_tensor(7, tensor, reqs, step_id=step_id, stream=s.cuda_stream, out_dtype=out_dtype,
                            summary_mask=summary_mask, keep_mask=keep_mask, row_index=row_index)
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert len(views) == seq_before + 1 and views[-1].seq == seq_before
        got = views[-1].bytes()
        s.synchronize()
    return got


def _case(B, tensor, reqs, *, seq, step_id, rank_tag=0, out_dtype=None, summary_mask=0, keep=None, index=None,
          out_bytes=4 << 20):
    reqs = np.asarray(reqs, dtype=np.uint32).reshape(-1, 5)
    s = torch.cuda.current_stream()
    km = None if keep is None else torch.tensor(keep, dtype=torch.uint8, device=DEV)
    ri = None if index is None else torch.tensor(index, dtype=torch.int32, device=DEV)
    od = {torch.bfloat16: 1, torch.float16: 2, torch.float32: 3}[tensor.dtype] if out_dtype is None else out_dtype
    out = torch.full((out_bytes,), POISON, dtype=torch.uint8, device=DEV)
    ub = B.observe_into(7, tensor, reqs, out, seq=seq, step_id=step_id, rank_tag=rank_tag, out_dtype=od,
                        summary_mask=summary_mask, keep_mask=km, row_index=ri, stream=s.cuda_stream)
    s.synchronize()
    host = out.cpu().numpy()
    size = int(host[48:56].view(np.uint64)[0])
    assert 64 <= size <= ub <= out_bytes and size % 64 == 0
    if keep is None:
        assert size == ub
    assert np.all(host[size:] == POISON), "bytes behind the record were written"
    rec = host[:size].copy()
    ref_ring = _via_ring(B, tensor, reqs, seq_before=seq, step_id=step_id, rank_tag=rank_tag, out_dtype=od,
                         summary_mask=summary_mask, keep_mask=km, row_index=ri)
    assert rec.size == ref_ring.size and np.array_equal(rec, ref_ring), "differs from dmi_observe's record"
    ref = orc.build_record(tensor.cpu(), reqs, seq=seq, step_id=step_id, point_id=7, out_dtype=od,
                           summary_mask=summary_mask, keep_mask=keep, row_index=index, rank_tag=rank_tag)
    compare_record(rec, ref, what="dmi_observe_into vs oracle")
    return size


def test_two_calls_in_a_row_the_second_smaller(B):
    big = prng.randn_bf16(5, 300 * 4096, DEV).reshape(300, 4096)
    # ragged selection, fp8 downcast, all three summaries, a keep vector: the general kernel
    reqs_big = [[10, 0, 0, 40, 1], [11, 40, 3, 30, 2], [12, 120, 0, 1, 1], [13, 130, 5, 50, 3], [14, 299, 0, 1, 1]]
    n1 = _case(B, big, reqs_big, seq=2, step_id=77, rank_tag=5, out_dtype=DT_FP8, summary_mask=7,
               keep=[1, 1, 0, 1, 1])
    # smaller input straight after: decode-shaped, 3 requests x 1 row x 256, raw bf16
    small = prng.randn_bf16(6, 40 * 256, DEV).reshape(40, 256)
    n2 = _case(B, small, [[1, 3, 0, 1, 1], [2, 17, 0, 1, 1], [3, 39, 0, 1, 1]], seq=0, step_id=78)
    assert n2 < n1
    # and a third one that lists several rows per request with no keep vector (row map behind the table)
    _case(B, small, [[1, 0, 1, 5, 2], [2, 20, 0, 7, 1]], seq=1, step_id=79, out_dtype=DT_FP16, summary_mask=5)


def test_limits_are_errors_not_launches(B):
    t = prng.randn_bf16(7, 64 * 128, DEV).reshape(64, 128)
    out = torch.full((4096,), POISON, dtype=torch.uint8, device=DEV)
    many = np.zeros((1025, 5), dtype=np.uint32)
    many[:, 3] = 1
    many[:, 4] = 1
    with pytest.raises(B.DmiError) as e:
        B.observe_into(1, t, many, out, seq=0, step_id=0)
    assert e.value.code == B.ERR_TOO_LARGE and "1024" in str(e.value)
    with pytest.raises(B.DmiError) as e:       # 64 rows x 256 B do not fit 4096 bytes
        B.observe_into(1, t, [[0, 0, 0, 64, 1]], out, seq=0, step_id=0)
    assert e.value.code == B.ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert bool((out == POISON).all())
