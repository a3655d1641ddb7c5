"""The test hooks of include/dmi_debug.h that the benchmark relies on: a capture launch timed by the
hardware's own start and end stamps is the same launch (same record), and the stamps make sense."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle as orc
from workloads import prng

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _event(hip):
    e = C.c_void_p()
    assert hip.hipEventCreate(C.byref(e)) == 0
    return e


@pytest.mark.parametrize("rows,elems", [(64, 4096), (3000, 4096)])     # decode-shaped kernel, general kernel
def test_a_timed_launch_is_the_same_launch(rows, elems):
    from paper_2605_11093_amd import binding as B
    B.lib()
    hip = C.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    hip.hipEventSynchronize.argtypes = [C.c_void_p]
    hip.hipEventDestroy.argtypes = [C.c_void_p]
    t = prng.randn_bf16(91, rows * elems, DEV).view(rows, elems)
    reqs = [(7, 0, 0, rows, 1)] if rows > 1024 else [(r, r, 0, 1, 1) for r in range(rows)]
    k0, k1 = _event(hip), _event(hip)
    with B.Ring(1 << 26, 1 << 26, max_reqs_per_observe=256) as ring:
        s = torch.cuda.current_stream()
        for seq in range(2):                     # the first launch timed, the second not: the hook is for one launch
            if seq == 0:
                B.time_next_launch(k0, k1)
            ring.observe_tensor(3, t, reqs, step_id=seq, stream=s.cuda_stream)
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert [v.seq for v in views] == [0, 1]
        for v in views:
            ref = orc.build_record(t.cpu(), reqs, seq=v.seq, step_id=v.seq, point_id=3, out_dtype=1)
            assert np.array_equal(v.bytes(), ref)
        assert hip.hipEventSynchronize(k1) == 0
        ms = C.c_float()
        assert hip.hipEventElapsedTime(C.byref(ms), k0, k1) == 0
        # a kernel of this size takes microseconds: more than nothing, far less than a millisecond
        assert 0.0005 < ms.value < 1.0, ms.value
        s.synchronize()
    hip.hipEventDestroy(k0)
    hip.hipEventDestroy(k1)
