"""The C ABI used from plain C (examples/c_client.c, built by build()): no Python and no
torch on the product side.  The records it writes must be the oracle's."""
import os
import subprocess

import numpy as np
import pytest

import oracle as orc
from oracle.decode import record_offsets
from workloads import prng
from _util import compare_record

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_client_writes_the_oracles_records(tmp_path):
    exe = os.path.join(ROOT, "examples", "c_client")
    if not os.path.exists(exe):         # normally built beforehand by __graft_entry__.build()
        import paper_2605_11093_amd as dmi
        from paper_2605_11093_amd import build as b
        dmi.lib()
        b.build_c_client()
    rows, elems = 48, 1024
    t = prng.randn_bf16(prng.sub_seed(41, 1), rows * elems).view(rows, elems)
    inp, out = tmp_path / "in.bin", tmp_path / "out.bin"
    t.view(dtype=__import__("torch").int16).numpy().tofile(inp)
    r = subprocess.run([exe, str(inp), str(rows), str(elems), str(out)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    got = np.fromfile(out, dtype=np.uint8)
    reqs = np.array([(100 + i, i * 7, 0, 1 + i % 3, 1) for i in range(6)], dtype=np.uint32)
    keep = np.array([1, 0, 1, 1, 0, 1], dtype=np.uint8)
    want = [orc.build_record(t, reqs, seq=0, step_id=40, point_id=1, out_dtype=1, summary_mask=5, rank_tag=7),
            orc.build_record(t, reqs, seq=1, step_id=40, point_id=2, out_dtype=4, rank_tag=7),
            orc.build_record(t, reqs, seq=2, step_id=41, point_id=3, out_dtype=1, summary_mask=5, keep_mask=keep,
                             rank_tag=7)]
    # dmi_observe_batch on the two halves of the tensor: the records of two single observes
    reqs2 = np.array([(200, 2, 0, 3, 3), (201, rows // 2 - 1, 0, 1, 1)], dtype=np.uint32)
    want += [orc.build_record(t[:rows // 2], reqs2, seq=3, step_id=42, point_id=4, out_dtype=2, summary_mask=2, rank_tag=7),
             orc.build_record(t[rows // 2:], reqs2, seq=4, step_id=42, point_id=5, out_dtype=2, summary_mask=2, rank_tag=7)]
    offs = record_offsets(got)
    assert [s for s, _, _ in offs] == [0, 1, 2, 3, 4]
    for (seq, off, n), w in zip(offs, want):
        compare_record(got[off:off + n], w, what=f"seq {seq}")
    assert "5 records" in r.stdout and "rows captured" in r.stdout
