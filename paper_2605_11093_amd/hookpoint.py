"""HookPoint front end (paper section 4.1): an nn.Module that can be put at any tensor
in a model's forward; reaching it launches one capture on the current stream and
returns the tensor itself.  No Python callback runs on the GPU's time line, no host
synchronisation happens, the tensor is neither modified nor retained.

Reaching a HookPoint is one call of the operator dmi::observe(x, hook), which is native code
(csrc/dmi_torch_op.cpp, built into libdmi_torch.so): it reads the tensor's address, layout and
current stream and calls the C ABI's dmi_observe.  This file only keeps the handles: the ring,
the point id, and the step context (request selection, step id) that the serving loop sets once
per forward step (the paper's prepare_step).  There is no Python implementation of the operator:
without the built library, making a HookPoint raises.

Under graph capture (StepContext.capture) a HookPoint adds its launch to a replayable
step (dmi_step_observe) instead, so the captures sit in the same graph as the model's own
kernels; StepContext.begin_replay / end_replay bracket each replay of that graph.
"""
from __future__ import annotations

import ctypes as C
import os
import weakref
from typing import Dict, Iterable, Optional

import numpy as np
import torch
from torch import nn

from . import binding as B

_TORCH_SO = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdmi_torch.so")
_native = None


def native():
    """Load libdmi_torch.so: registers the operator dmi::observe with PyTorch and gives the handle
    functions.  Raises if it has not been built."""
    global _native
    if _native is not None:
        return _native
    B.lib()                                     # libdmi.so first: the operator library links against it
    if not os.path.exists(_TORCH_SO):
        raise ImportError(f"{_TORCH_SO} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    torch.ops.load_library(_TORCH_SO)
    L = C.CDLL(_TORCH_SO)
    L.dmi_torch_ctx_create.restype = C.c_int32
    L.dmi_torch_ctx_set.argtypes = [C.c_int32, C.c_uint64, C.c_void_p, C.c_uint32, C.c_void_p]
    L.dmi_torch_ctx_capture.argtypes = [C.c_int32, C.c_void_p]
    L.dmi_torch_ctx_nodes.argtypes = [C.c_int32, C.POINTER(C.c_uint32), C.c_uint32]
    L.dmi_torch_ctx_nodes.restype = C.c_uint32
    L.dmi_torch_hook_create.argtypes = [C.c_void_p, C.c_uint32, C.c_int32, C.c_uint32, C.c_int32]
    L.dmi_torch_hook_create.restype = C.c_int32
    L.dmi_torch_hook_destroy.argtypes = [C.c_int32]

    @torch.library.register_fake("dmi::observe")
    def _observe_fake(x, hook):                 # shape propagation for tracing: no result
        return None

    _native = L
    return L


class StepContext:
    """What every HookPoint of a forward step shares: which rows belong to which
    request, the step id, an optional keep vector (device address).  The values live in the
    operator library, where the hooks read them; this object is the handle."""

    def __init__(self):
        self._id = native().dmi_torch_ctx_create()
        self._reqs: Optional[np.ndarray] = None
        self.step_id = 0
        self.keep_mask_dev = 0
        self.step: Optional[B.Step] = None          # set while / after a graph capture
        self._keep_tensor = None

    def _push(self):
        r = self._reqs
        B._check(native().dmi_torch_ctx_set(self._id, self.step_id, None if r is None else r.ctypes.data,
                                            0 if r is None else r.shape[0], self.keep_mask_dev or None))

    @property
    def reqs(self) -> Optional[np.ndarray]:
        return self._reqs

    @reqs.setter
    def reqs(self, value):
        """None: no step prepared, hooks launch nothing."""
        self._reqs = None if value is None else np.ascontiguousarray(np.asarray(value, dtype=np.uint32).reshape(-1, 5))
        self._push()

    def prepare_step(self, step_id: int, reqs, keep_mask_dev: int = 0):
        self.step_id = int(step_id)
        self.keep_mask_dev = int(keep_mask_dev)
        self.reqs = reqs

    @property
    def _nodes(self):
        n = native().dmi_torch_ctx_nodes(self._id, None, 0)
        out = (C.c_uint32 * max(n, 1))()
        native().dmi_torch_ctx_nodes(self._id, out, n)
        return list(out[:n])

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
                ctx._keep_tensor = keep_mask
                ctx.prepare_step(ctx.step_id, reqs, 0 if keep_mask is None else keep_mask.data_ptr())
                ctx.step.capture_begin()
                B._check(native().dmi_torch_ctx_capture(ctx._id, ctx.step._h))
                return ctx.step

            def __exit__(self_inner, *exc):
                B._check(native().dmi_torch_ctx_capture(ctx._id, None))
                ctx.step.seal()
                return False

        return _Capture()

    def begin_replay(self, step_id: int, stream: int, reqs=None, allow=()) -> int:
        """Before replaying the captured graph on `stream`: optional new batch composition
        (same number of requests), then the step's policy gate and parameter upload."""
        if reqs is not None:
            ra = np.ascontiguousarray(np.asarray(reqs, dtype=np.uint32).reshape(-1, 5))
            if not np.array_equal(ra, self._reqs):
                nodes = self._nodes
                if nodes:
                    self.step.update(nodes[0], ra)          # all hook points share the step's one table
                self.reqs = ra
        return self.step.begin(step_id, stream, allow=allow)

    def end_replay(self, stream: int):
        self.step.end(stream)


class HookPoint(nn.Module):
    """Identity module that observes its input.  `enabled=False` makes it a plain
    identity: nothing is launched (hook filtering).  out_dtype None = store the source dtype."""

    def __init__(self, ring: B.Ring, point_id: int, ctx: StepContext, *, out_dtype: Optional[int] = None,
                 summary_mask: int = 0, enabled: bool = True, name: str = ""):
        super().__init__()
        self.ring, self.point_id, self.ctx = ring, int(point_id), ctx
        self.out_dtype, self.summary_mask, self.enabled, self.hook_name = out_dtype, summary_mask, enabled, name
        hid = native().dmi_torch_hook_create(ring._h, self.point_id, -1 if out_dtype is None else int(out_dtype),
                                             int(summary_mask), ctx._id)
        B._check(hid)
        self._hook_id = hid
        weakref.finalize(self, native().dmi_torch_hook_destroy, hid)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if not self.enabled:            # hook filtering: a disabled hook is not in the graph at all
            return x
        if self.ring._h is None:
            raise B.DmiError(B.ERR_CLOSED, "HookPoint reached after its ring was destroyed")
        torch.ops.dmi.observe(x, self._hook_id)
        return x


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
