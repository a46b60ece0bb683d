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

    def run(self, args, stream=None):
        B.bcast_dual_forward(self.op_id, args, self.outs, self.partials, self.branch, stream)
        return self


@dataclass
class BackwardBuffers:
    grads: List = field(default_factory=list)      # N_d tensors in their argument's shape
    workspace: Optional[object] = None

    def run(self, adjoints, partials, stream=None):
        B.bcast_dual_backward(adjoints, partials, self.grads, self.workspace, stream)
        return self


def unified_shape(args):
    nd = max(a.dim() for a in args)
    shape = [1] * nd
    for a in args:
        for d in range(a.dim()):
            if a.shape[d] != 1:
                shape[d] = a.shape[d]
    return tuple(shape)


def alloc_forward(op_name: str, args, want_branch: bool = False, want_partials: bool = True) -> ForwardBuffers:
    import torch
    op_id = B.bcast_op_lookup(op_name)
    n, m, mask, _ = B.bcast_op_info(op_id)
    nd = n - bin(mask).count("1")
    shape = unified_shape(args)
    kw = dict(dtype=args[0].dtype, device=args[0].device)
    outs = [torch.empty(shape, **kw) for _ in range(m)]
    parts = [torch.empty(shape, **kw) for _ in range(m * nd)] if want_partials else None
    br = torch.empty(shape, dtype=torch.uint8, device=args[0].device) if want_branch else None
    return ForwardBuffers(op_id, outs, parts, br)


def alloc_backward(adjoints, partials, grad_shapes) -> BackwardBuffers:
    import torch
    kw = dict(dtype=adjoints[0].dtype, device=adjoints[0].device)
    grads = [torch.empty(tuple(s), **kw) for s in grad_shapes]
    nbytes = B.bcast_dual_backward_workspace(adjoints, partials, grads)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=adjoints[0].device) if nbytes else None
    return BackwardBuffers(grads, ws)
