"""The fused broadcast as ONE node of a reverse-mode program (Sec. 2.2.3 of arXiv 1810.08297:
forward mode inside, reverse mode outside).  `broadcast(op, *args)` runs the dual-number
forward kernel and hands torch.autograd a node whose backward is the library's adjoint x
partial kernel with its broadcast-dim reductions -- or, with planes="none", the kernel that
evaluates the dual numbers again (the alternative at the end of Sec. 2.2.3).

Marshalling only: every number is computed by the library's kernels.  Arguments follow
torch's broadcasting rule (shapes aligned at the LAST dim, missing leading dims count as 1);
the C ABI itself pads at the end, as the paper's Eq. 1 does, so full-rank views are passed.
"""
from __future__ import annotations

import torch
from torch.autograd.function import once_differentiable

from . import binding as B
from .helpers import alloc_forward

_MODES = ("all", "lean", "none")


def _full_rank(t, nd):
    return t[(None,) * (nd - t.dim()) + (Ellipsis,)] if t.dim() < nd else t


class _BroadcastNode(torch.autograd.Function):
    @staticmethod
    def forward(ctx, op_name, planes, *args):
        op_id = B.bcast_op_lookup(op_name)
        n_args, n_out, mask, _ = B.bcast_op_info(op_id)
        if len(args) != n_args:
            raise ValueError(f"{op_name} takes {n_args} arguments, got {len(args)}")
        nd = max(a.dim() for a in args)
        full = [_full_rank(a, nd) for a in args]
        fb = alloc_forward(op_name, full, want_partials=planes != "none", lean=planes == "lean")
        fb.run(full)
        ctx.op_id, ctx.mask, ctx.planes, ctx.nd = op_id, mask, planes, nd
        ctx.arg_shapes = [tuple(a.shape) for a in args]
        if planes == "none":
            ctx.save_for_backward(*args)
        else:
            ctx.partials, ctx.slab = fb.partials, fb.slab  # cached until the reverse pass reaches this node
        return tuple(fb.outs)

    @staticmethod
    @once_differentiable
    def backward(ctx, *adjoints):
        adj = [a if a.is_contiguous() else a.contiguous() for a in adjoints]
        n_args = len(ctx.arg_shapes)
        diff = [j for j in range(n_args) if not (ctx.mask >> j) & 1]
        full_shape = lambda j: (1,) * (ctx.nd - len(ctx.arg_shapes[j])) + ctx.arg_shapes[j]
        grads = [torch.empty(full_shape(j), dtype=adj[0].dtype, device=adj[0].device) if ctx.needs_input_grad[2 + j] else None
                 for j in diff]
        if any(g is not None for g in grads):
            if ctx.planes == "none":
                full = [_full_rank(a, ctx.nd) for a in ctx.saved_tensors]
                nbytes = B.bcast_dual_backward_recompute_workspace(ctx.op_id, full, adj, grads)
                ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=adj[0].device) if nbytes else None
                B.bcast_dual_backward_recompute(ctx.op_id, full, adj, grads, ws)
            else:
                nbytes = B.bcast_dual_backward_workspace(adj, ctx.partials, grads)
                ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=adj[0].device) if nbytes else None
                B.bcast_dual_backward(adj, ctx.partials, grads, ws)
        out = [None, None] + [None] * n_args
        for g, j in zip(grads, diff):
            if g is not None:
                out[2 + j] = g.reshape(ctx.arg_shapes[j])
        return tuple(out)


def broadcast(op_name: str, *args, planes: str = "lean"):
    """b.(X1..XN) for an op of the library's table, differentiable by torch.autograd.

    planes: "all" = every partial plane is cached between the passes; "lean" (default) = planes
    the op declares identical are stored once and always-zero planes not at all; "none" = nothing
    is cached and the reverse pass evaluates the dual numbers again.  Returns one tensor, or a
    tuple for ops with several outputs."""
    if planes not in _MODES:
        raise ValueError(f"planes must be one of {_MODES}")
    outs = _BroadcastNode.apply(op_name, planes, *args)
    return outs[0] if len(outs) == 1 else outs
