"""Device-buffer allocation around the C-ABI calls (PyTorch = memory and streams only)."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

from . import binding as B


@dataclass
class ForwardBuffers:
    op_id: int
    outs: List = field(default_factory=list)       # M tensors of the unified shape
    partials: List = field(default_factory=list)   # M*N_d planes, index i*N_d + jd
    branch: Optional[object] = None                # uint8, unified shape
    slab: Optional[object] = None                  # keeps the memory of outs/partials alive
    options: Optional[B.Options] = None            # bcast_dual_options of every call (None = defaults)

    def run(self, args, stream=None):
        B.bcast_dual_forward(self.op_id, args, self.outs, self.partials, self.branch, stream, self.options)
        return self

    def prepare(self, args):
        """Marshal the call once; the returned object's launch() only enqueues the kernel."""
        return B.PreparedForward(self.op_id, args, self.outs, self.partials, self.branch, self.options)


@dataclass
class BackwardBuffers:
    grads: List = field(default_factory=list)      # N_d tensors in their argument's shape
    workspace: Optional[object] = None
    slab: Optional[object] = None
    options: Optional[B.Options] = None            # the workspace was sized for these

    def run(self, adjoints, partials, stream=None):
        B.bcast_dual_backward(adjoints, partials, self.grads, self.workspace, stream, self.options)
        return self

    def prepare(self, adjoints, partials):
        return B.PreparedBackward(adjoints, partials, self.grads, self.workspace, self.options)


def unified_shape(args):
    nd = max(a.dim() for a in args)
    shape = [1] * nd
    for a in args:
        for d in range(a.dim()):
            if a.shape[d] != 1:
                shape[d] = a.shape[d]
    return tuple(shape)


def _numel(shape):
    n = 1
    for s in shape:
        n *= int(s)
    return n


def alloc_planes(shapes, dtype, device, staggered: bool = True, layout: Optional[str] = None):
    """Tensors of the given shapes.  The ones that share the largest size are carved out of one slab:
    layout "staggered" (the default; `staggered=False` = "plain"): each a contiguous plane, in the
    library's staggered layout (bcast_dual_slab_layout); layout "interleaved": the planes interleaved
    along their first dim -- row r of plane k follows row r of plane k - 1 -- so that a block that
    writes one row step of every plane writes one contiguous run (views with a row stride of
    n_planes x the row length; measured faster where some twenty planes that exceed the memory-side
    cache are streamed at once).  The rest are ordinary allocations.  Returns (tensors, slab)."""
    import torch
    layout = layout or ("staggered" if staggered else "plain")
    if layout not in ("staggered", "plain", "interleaved"):
        raise ValueError(f"unknown layout {layout!r}")
    es = torch.empty((), dtype=dtype).element_size()
    shapes = [tuple(int(x) for x in s) for s in shapes]
    big = max((_numel(s) for s in shapes), default=0)
    idx = [k for k, s in enumerate(shapes) if _numel(s) == big] if layout != "plain" and big > 0 else []
    out = [None] * len(shapes)
    slab = None
    if idx and layout == "interleaved" and len({shapes[k] for k in idx}) == 1 and len(shapes[idx[0]]) >= 2:
        shp = shapes[idx[0]]
        slab = torch.empty((shp[0], len(idx)) + shp[1:], dtype=dtype, device=device)
        for n, k in enumerate(idx):
            out[k] = slab[:, n]
    elif idx:
        total, offs = B.bcast_dual_slab_layout(big * es, len(idx))
        slab = torch.empty(total, dtype=torch.uint8, device=device)
        for n, k in enumerate(idx):
            out[k] = slab[offs[n]: offs[n] + big * es].view(dtype).view(shapes[k])
    for k, s in enumerate(shapes):
        if out[k] is None:
            out[k] = torch.empty(s, dtype=dtype, device=device)
    return out, slab


def to_slab(tensors, staggered: bool = True, layout: Optional[str] = None):
    """Copy tensors (same dtype and device) into freshly allocated planes of the given layout (see alloc_planes)."""
    out, slab = alloc_planes([t.shape for t in tensors], tensors[0].dtype, tensors[0].device, staggered, layout)
    for o, t in zip(out, tensors):
        o.copy_(t)
    return out, slab


def alloc_forward(op_name: str, args, want_branch: bool = False, want_partials: bool = True,
                  staggered: bool = True, lean: bool = False, options: Optional[B.Options] = None,
                  layout: Optional[str] = None) -> ForwardBuffers:
    """``lean``: planes the op table declares identical share one buffer and planes it declares
    zero are left out (None); forward and backward give the same results with fewer bytes moved."""
    import torch
    op_id = B.bcast_op_lookup(op_name)
    n, m, mask, _ = B.bcast_op_info(op_id)
    nd = n - bin(mask).count("1")
    shape = unified_shape(args)
    br = torch.empty(shape, dtype=torch.uint8, device=args[0].device) if want_branch else None
    if not want_partials:
        outs, slab = alloc_planes([shape] * m, args[0].dtype, args[0].device, staggered, layout)
        return ForwardBuffers(op_id, outs, None, br, slab, options)
    alias = B.bcast_op_plane_alias(op_id) if lean else list(range(m * nd))
    own = [k for k in range(m * nd) if alias[k] == k]
    planes, slab = alloc_planes([shape] * (m + len(own)), args[0].dtype, args[0].device, staggered, layout)
    store = dict(zip(own, planes[m:]))
    parts = [None if alias[k] < 0 else store[alias[k]] for k in range(m * nd)]
    return ForwardBuffers(op_id, planes[:m], parts, br, slab, options)


def alloc_backward(adjoints, partials, grad_shapes, staggered: bool = True,
                   options: Optional[B.Options] = None, layout: Optional[str] = None) -> BackwardBuffers:
    import torch
    grads, slab = alloc_planes(grad_shapes, adjoints[0].dtype, adjoints[0].device, staggered, layout)
    nbytes = B.bcast_dual_backward_workspace(adjoints, partials, grads, options)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=adjoints[0].device) if nbytes else None
    return BackwardBuffers(grads, ws, slab, options)


def alloc_recompute(op_id: int, args, adjoints, grad_shapes, staggered: bool = True,
                    options: Optional[B.Options] = None, layout: Optional[str] = None) -> BackwardBuffers:
    """Gradient buffers and workspace for bcast_dual_backward_recompute."""
    import torch
    grads, slab = alloc_planes(grad_shapes, adjoints[0].dtype, adjoints[0].device, staggered, layout)
    nbytes = B.bcast_dual_backward_recompute_workspace(op_id, args, adjoints, grads, options)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=adjoints[0].device) if nbytes else None
    return BackwardBuffers(grads, ws, slab, options)


class LaunchTimer:
    """A pair of HIP events for the `start_event` / `stop_event` fields of bcast_dual_options:
    pass `timer.options(base)` to the call whose main kernel is to be timed, read `ms()` after
    the stream has been synchronised."""

    _hip = None

    def __init__(self):
        import ctypes
        if LaunchTimer._hip is None:
            LaunchTimer._hip = ctypes.CDLL("libamdhip64.so")
        self._start, self._stop = ctypes.c_void_p(), ctypes.c_void_p()
        for ev in (self._start, self._stop):
            if LaunchTimer._hip.hipEventCreate(ctypes.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")

    def options(self, base: Optional[B.Options] = None) -> B.Options:
        """`base` (or the defaults) with this timer's events in it."""
        return (base or B.Options()).replace(start_event=self._start.value, stop_event=self._stop.value)

    def ms(self) -> float:
        import ctypes
        out = ctypes.c_float()
        rc = LaunchTimer._hip.hipEventElapsedTime(ctypes.byref(out), self._start, self._stop)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(out.value)

    def __del__(self):
        try:
            for ev in (self._start, self._stop):
                LaunchTimer._hip.hipEventDestroy(ev)
        except Exception:
            pass
