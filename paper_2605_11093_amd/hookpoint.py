"""HookPoint front end (paper section 4.1): an nn.Module that can be put at any tensor
in a model's forward; reaching it launches one capture on the current stream and
returns the tensor itself.  No Python callback runs on the GPU's time line, no host
synchronisation happens, the tensor is neither modified nor retained.

The work is the C ABI's dmi_observe; this file only finds the arguments: the ring, the
point id, and the step context (request selection, step id) that the serving loop sets
once per forward step (the paper's prepare_step).

Under graph capture (StepContext.capture) a HookPoint adds its launch to a replayable
step (dmi_step_observe) instead, so the captures sit in the same graph as the model's own
kernels; StepContext.begin_replay / end_replay bracket each replay of that graph.
"""
from __future__ import annotations

import weakref
from typing import Dict, Iterable, Optional

import numpy as np
import torch
from torch import nn

from . import binding as B


class StepContext:
    """What every HookPoint of a forward step shares: which rows belong to which
    request, the step id, an optional keep vector (device address)."""

    def __init__(self):
        self.reqs: Optional[np.ndarray] = None
        self.step_id = 0
        self.keep_mask_dev = 0
        self.step: Optional[B.Step] = None          # set while / after a graph capture
        self._capturing = False
        self._nodes: list = []
        self._keep_tensor = None

    def prepare_step(self, step_id: int, reqs, keep_mask_dev: int = 0):
        self.reqs = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
        self.step_id = int(step_id)
        self.keep_mask_dev = int(keep_mask_dev)

    # -- graph capture and replay ------------------------------------------
    def capture(self, ring: B.Ring, reqs, *, max_observes: int = 64, keep_mask=None):
        """Context manager around the caller's graph capture of one forward step:

            with ctx.capture(ring, reqs, keep_mask=mask_tensor):
                with torch.cuda.graph(g):
                    y = model(static_x)

        reqs is the selection the step is captured with (its shape stays; contents may be
        replaced per replay); keep_mask an optional uint8 device tensor that the caller
        rewrites between replays."""
        ctx = self

        class _Capture:
            def __enter__(self_inner):
                ctx.step = B.Step(ring, max_observes)
                ctx.reqs = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
                ctx.keep_mask_dev = 0 if keep_mask is None else keep_mask.data_ptr()
                ctx._keep_tensor = keep_mask
                ctx._nodes = []
                ctx.step.capture_begin()
                ctx._capturing = True
                return ctx.step

            def __exit__(self_inner, *exc):
                ctx._capturing = False
                ctx.step.seal()
                return False

        return _Capture()

    def begin_replay(self, step_id: int, stream: int, reqs=None, allow=()) -> int:
        """Before replaying the captured graph on `stream`: optional new batch composition
        (same number of requests), then the step's policy gate and parameter upload."""
        if reqs is not None:
            ra = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
            if not np.array_equal(ra, self.reqs):
                if self._nodes:
                    self.step.update(self._nodes[0], ra)    # all hook points share the step's one table
                self.reqs = ra
        return self.step.begin(step_id, stream, allow=allow)

    def end_replay(self, stream: int):
        self.step.end(stream)


# The custom-operator layer (paper section 4.1): reaching a HookPoint is one call of the
# operator dmi::observe(x, hook), so a traced / compiled model carries the capture as an
# ordinary node of its graph instead of breaking at a Python callback.  The operator is
# declared as writing its input (it writes nothing): that keeps compilers from dropping a
# call whose result nobody uses, and from moving it across other uses of the tensor.
_HOOKS: "weakref.WeakValueDictionary[int, HookPoint]" = weakref.WeakValueDictionary()
_next_hook_id = 0
_op_registered = False


def _register_op():
    global _op_registered
    if _op_registered:
        return
    _op_registered = True

    @torch.library.custom_op("dmi::observe", mutates_args=("x",))
    def _observe(x: torch.Tensor, hook: int) -> None:
        _HOOKS[hook]._launch(x)


class HookPoint(nn.Module):
    """Identity module that observes its input.  `enabled=False` makes it a plain
    identity: nothing is launched (hook filtering)."""

    def __init__(self, ring: B.Ring, point_id: int, ctx: StepContext, *, out_dtype: Optional[int] = None,
                 summary_mask: int = 0, enabled: bool = True, name: str = ""):
        super().__init__()
        self.ring, self.point_id, self.ctx = ring, int(point_id), ctx
        self.out_dtype, self.summary_mask, self.enabled, self.hook_name = out_dtype, summary_mask, enabled, name
        _register_op()
        global _next_hook_id
        _next_hook_id += 1
        self._hook_id = _next_hook_id
        _HOOKS[self._hook_id] = self

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if not self.enabled:            # hook filtering: a disabled hook is not in the graph at all
            return x
        torch.ops.dmi.observe(x, self._hook_id)
        return x

    def _launch(self, x: torch.Tensor) -> None:
        if self.ctx.reqs is None:
            return
        t = x if x.dim() == 2 else x.reshape(-1, x.shape[-1])      # [tokens, features] view, no copy
        if t.stride(-1) != 1 or t.data_ptr() != x.data_ptr():
            raise ValueError("HookPoint needs a tensor whose rows are contiguous in memory")
        dt = B._torch_dtype_code(t)
        if self.ctx._capturing:
            node = self.ctx.step.observe_tensor(self.point_id, t, self.ctx.reqs,
                                                stream=torch.cuda.current_stream(x.device).cuda_stream,
                                                out_dtype=dt if self.out_dtype is None else self.out_dtype,
                                                summary_mask=self.summary_mask, keep_mask=self.ctx._keep_tensor)
            if node >= 0:
                self.ctx._nodes.append(node)
            return
        self.ring.observe(self.point_id, t.data_ptr(), dt, tuple(t.shape), tuple(t.stride()), self.ctx.reqs,
                          step_id=self.ctx.step_id, stream=torch.cuda.current_stream(x.device).cuda_stream,
                          out_dtype=dt if self.out_dtype is None else self.out_dtype,
                          summary_mask=self.summary_mask, keep_mask_dev=self.ctx.keep_mask_dev,
                          allow=())


def install_hookpoints(model: nn.Module, ring: B.Ring, ctx: StepContext, where: Dict[str, int],
                       enabled: Optional[Iterable[str]] = None, **kw) -> Dict[str, HookPoint]:
    """Wrap the named sub-modules so that their output passes through a HookPoint.
    where: sub-module path -> point id.  enabled: the hook set to switch on (default all)."""
    made = {}
    on = None if enabled is None else set(enabled)
    for path, pid in where.items():
        parent_path, _, leaf = path.rpartition(".")
        parent = model.get_submodule(parent_path) if parent_path else model
        inner = getattr(parent, leaf)
        hp = HookPoint(ring, pid, ctx, enabled=on is None or path in on, name=path, **kw)
        setattr(parent, leaf, nn.Sequential(inner, hp))
        made[path] = hp
    return made
