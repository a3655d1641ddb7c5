"""HookPoint front end: observing does not change the model's output, disabled hooks
launch nothing, and what is captured equals the oracle's record of the same tensor."""
import numpy as np
import pytest
import torch
from torch import nn

import oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


class Block(nn.Module):
    def __init__(self, d):
        super().__init__()
        self.ln = nn.LayerNorm(d)
        self.up = nn.Linear(d, 4 * d)
        self.down = nn.Linear(4 * d, d)

    def forward(self, x):
        return x + self.down(torch.nn.functional.gelu(self.up(self.ln(x))))


def test_hookpoints_capture_without_changing_the_forward():
    from paper_2605_11093_amd import binding as B
    from paper_2605_11093_amd.hookpoint import HookPoint, StepContext, install_hookpoints
    torch.manual_seed(0)
    d, T = 256, 24
    model = nn.Sequential(*[Block(d) for _ in range(3)]).to(DEV).to(torch.bfloat16).eval()
    x = torch.randn(T, d, device=DEV).to(torch.bfloat16)
    with torch.no_grad():
        plain = model(x).clone()
    captured = {}
    with B.Ring(1 << 20, 1 << 20) as ring:
        ctx = StepContext()
        hooks = install_hookpoints(model, ring, ctx, {"0": 10, "1.up": 11, "2": 12}, enabled=["0", "1.up"],
                                   summary_mask=5)
        # spy on the tensors that reach the enabled hooks (test only; the hook itself keeps nothing)
        for name, hp in hooks.items():
            hp.register_forward_pre_hook(lambda m, a, n=name: captured.__setitem__(n, a[0].detach().clone()))
        reqs = [(70, 0, 20, 4, 1), (71, 0, 3, 2, 5)]       # rows 20..23 and rows 3, 8
        ctx.prepare_step(5, reqs)
        with torch.no_grad():
            hooked = model(x)
        assert torch.equal(hooked, plain)
        ring.drain(B.DRAIN_FLUSH)
        views = ring.poll_host()
        assert [v.seq for v in views] == [0, 1]            # the disabled hook launched nothing
        st = ring.get_stats()
        assert st.observed_calls == 2 and st.launched_records == 2
        from _util import compare_record
        for v, (name, pid) in zip(views, (("0", 10), ("1.up", 11))):
            t = captured[name].reshape(-1, captured[name].shape[-1]).cpu()
            ref = orc.build_record(t, reqs, seq=v.seq, step_id=5, point_id=pid, out_dtype=1, summary_mask=5)
            compare_record(v.bytes(), ref)


def test_hookpoints_inside_a_captured_graph():
    """The model's forward, HookPoints included, captured once and replayed: every replay's
    records equal the oracle's records of the tensors that replay produced."""
    from paper_2605_11093_amd import binding as B
    from paper_2605_11093_amd.hookpoint import StepContext, install_hookpoints
    from _util import compare_record
    torch.manual_seed(1)
    d, T = 256, 16
    model = nn.Sequential(*[Block(d) for _ in range(3)]).to(DEV).to(torch.bfloat16).eval()
    static_x = torch.zeros(T, d, device=DEV, dtype=torch.bfloat16)
    keep = torch.ones(T, dtype=torch.uint8, device=DEV)
    live = {}
    with B.Ring(1 << 20, 1 << 20) as ring:
        ctx = StepContext()
        hooks = install_hookpoints(model, ring, ctx, {"0": 10, "1.up": 11, "2": 12}, enabled=["0", "1.up", "2"],
                                   summary_mask=5)
        ring.point_enable(12, False)                # filtered out: not part of the graph
        # the tensors that reach the hooks live in the graph's memory pool; holding them keeps
        # their memory from being reused inside the graph, so they can be read after a replay
        for name, hp in hooks.items():
            hp.register_forward_pre_hook(lambda m, a, n=name: live.__setitem__(n, a[0]))
        reqs0 = [(100 + i, i, 0, 1, 1) for i in range(T)]
        with torch.no_grad():
            model(static_x)                         # warm-up outside the capture (library set-up, no hooks fire:
            torch.cuda.synchronize()                # no step prepared yet)
        assert ring.get_stats().launched_records == 0
        g = torch.cuda.CUDAGraph()
        with ctx.capture(ring, reqs0, keep_mask=keep):
            with torch.cuda.graph(g), torch.no_grad():
                model(static_x)
        s = torch.cuda.current_stream()
        seq = 0
        for step in range(5):
            x = torch.randn(T, d, device=DEV).to(torch.bfloat16)
            static_x.copy_(x)
            mask = (np.arange(T) % 3 != step % 3).astype(np.uint8) if step else np.ones(T, np.uint8)
            keep.copy_(torch.from_numpy(mask))
            reqs = [(1000 * step + i, i, 0, 1, 1) for i in range(T)]
            assert ctx.begin_replay(step, s.cuda_stream, reqs=reqs) == B.OK
            g.replay()
            ctx.end_replay(s.cuda_stream)
            s.synchronize()
            ring.drain(B.DRAIN_FLUSH)
            views = ring.poll_host()
            assert [v.seq for v in views] == [seq, seq + 1]
            for v, (name, pid) in zip(views, (("0", 10), ("1.up", 11))):
                t = live[name].reshape(-1, live[name].shape[-1]).cpu()
                ref = orc.build_record(t, reqs, seq=v.seq, step_id=step, point_id=pid, out_dtype=1, summary_mask=5,
                                       keep_mask=mask)
                compare_record(v.bytes(), ref)
            ring.release_host(views[-1].seq)
            seq += 2
        torch.cuda.synchronize()
        ctx.step.destroy()


def test_hookpoints_survive_compilation_as_graph_nodes():
    """torch.compile traces the model into one graph (no break at the hooks); the captures
    are nodes of that graph and still fire once per forward."""
    from paper_2605_11093_amd import binding as B
    from paper_2605_11093_amd.hookpoint import StepContext, install_hookpoints
    from _util import compare_record
    torch.manual_seed(2)
    d, T = 256, 12
    model = nn.Sequential(*[Block(d) for _ in range(2)]).to(DEV).to(torch.bfloat16).eval()
    live = {}
    with B.Ring(1 << 20, 1 << 20) as ring:
        ctx = StepContext()
        hooks = install_hookpoints(model, ring, ctx, {"0": 3, "1": 4})
        for name, hp in hooks.items():
            hp.register_forward_pre_hook(lambda m, a, n=name: live.__setitem__(n, a[0].detach().clone()))
        compiled = torch.compile(model, backend="aot_eager", fullgraph=True)
        reqs = [(5, 0, 2, 3, 4)]                        # rows 2, 6, 10
        seq = 0
        for step in range(3):
            x = torch.randn(T, d, device=DEV).to(torch.bfloat16)
            ctx.prepare_step(step, reqs)
            with torch.no_grad():
                y = compiled(x)
                ctx.reqs = None                         # the reference forward below must not capture
                ref_y = model(x)
            assert torch.equal(y, ref_y)
            ring.drain(B.DRAIN_FLUSH)
            views = ring.poll_host()
            assert [v.seq for v in views] == [seq, seq + 1]
            for v, (name, pid) in zip(views, (("0", 3), ("1", 4))):
                t = live[name].reshape(-1, d).cpu()
                compare_record(v.bytes(), orc.build_record(t, reqs, seq=v.seq, step_id=step, point_id=pid, out_dtype=1))
            ring.release_host(views[-1].seq)
            seq += 2


def test_hookpoint_operator_reads_layouts_and_refuses_what_it_cannot_view():
    """The native operator sees a tensor of any rank as [tokens, features] without a copy: leading
    dimensions that collapse into evenly spaced rows are fine (a batch dimension, a step through the
    tokens, a row pitch wider than the features); rows that are not evenly spaced, or whose elements
    are not contiguous, are refused; so is a hook whose ring is gone."""
    from paper_2605_11093_amd import binding as B
    from paper_2605_11093_amd.hookpoint import HookPoint, StepContext
    from workloads import prng
    Bt, T, E = 3, 10, 512
    x = prng.randn_bf16(77, Bt * T * E, DEV).view(Bt, T, E)
    cases = [
        ("batch of sequences", x, x.reshape(-1, E)),
        ("every second token", x[:, ::2, :], x[:, ::2, :].reshape(-1, E)),
        ("half of the features", x[0, :, :E // 2], x[0, :, :E // 2]),
        ("one sequence, kept 3-d", x[1:2], x[1]),
        ("a vector", x[2, 3], x[2, 3].reshape(1, E)),
    ]
    ring = B.Ring(1 << 22, 1 << 22)
    ctx = StepContext()
    hook = HookPoint(ring, 9, ctx, summary_mask=4)
    seq = 0
    with torch.no_grad():
        for what, view, rows in cases:
            n = rows.shape[0]
            reqs = [(1, 0, 0, n, 1)] if n < 4 else [(1, 0, 1, n // 2, 2), (2, 0, n - 1, 1, 1)]
            ctx.prepare_step(seq, reqs)
            y = hook(view)
            assert y is view
            ring.drain(B.DRAIN_FLUSH)
            (v,) = ring.poll_host()
            ref = orc.build_record(rows.contiguous().cpu(), reqs, seq=seq, step_id=seq, point_id=9, out_dtype=1,
                                   summary_mask=4)
            assert np.array_equal(v.bytes(), ref), what
            ring.release_host(v.seq)
            seq += 1
        ctx.prepare_step(seq, [(1, 0, 0, 2, 1)])
        for bad in (x[:, :T - 1, :], x.transpose(1, 2), x[0].t()):
            with pytest.raises(RuntimeError):
                hook(bad)
        with pytest.raises(RuntimeError):
            hook(x.to(torch.float64))
        assert ring.get_stats().launched_records == seq          # the refused calls launched nothing
        ctx.reqs = None
        hook(x)                                                   # no step prepared: a plain identity
        assert ring.get_stats().observed_calls == seq
        torch.cuda.synchronize()
        ring.destroy()
        ctx.prepare_step(seq, [(1, 0, 0, 2, 1)])
        with pytest.raises(B.DmiError):
            hook(x)
