"""Unfused reverse-mode comparison points (they stand in for the paper's per-primitive graph
baselines, Sec. 3.2.1 / 3.2.2 / 3.4): the same scalar functions as one kernel per primitive,
every branch computed for every element and chosen with a select, differentiated by plain
reverse mode.  Two forms: `UnfusedPrimitives` drives the library's own per-primitive HIP kernels
(bcast_unfused_step); `UnfusedStep` is the same chain on PyTorch's elementwise kernels and
torch.autograd.  NOT part of the product path: `bench.py --unfused-baseline` times both next to
the fused kernels, and GPU tests check that they compute the same function.
"""
from __future__ import annotations

import torch


def _hmlstm_update(f, i, o, g, c, h, z, zb, bf, bi, bo, bg):
    si, tg = torch.sigmoid(i + bi), torch.tanh(g + bg)
    flush = si * tg
    update = torch.sigmoid(f + bf) * c + flush
    is_flush = z == 1
    is_copy = (z == 0) & (zb == 0)
    cn = torch.where(is_flush, flush, torch.where(is_copy, c, update))
    hn = torch.where(is_copy & ~is_flush, h, torch.sigmoid(o + bo) * torch.tanh(cn))
    return cn, hn


def _update_c(c, f, i, g, z1, z2):
    flush = torch.sigmoid(i) * torch.tanh(g)
    update = torch.sigmoid(f) * c + flush
    return (torch.where(z1 == 1, flush, torch.where((z1 == 0) & (z2 == 0), c, update)),)


def _tanh_xy_b(x, y, b):
    return (torch.tanh(x * y + b),)


def _branchy5(a, b, r, s, t):
    return (torch.where(a + s > t, torch.exp(-a) * b + r, torch.log1p(a * a) * r - s),)


FUNCTIONS = {"hmlstm_update": (_hmlstm_update, (6, 7)), "update_c": (_update_c, (4, 5)),
             "tanh_xy_b": (_tanh_xy_b, ()), "branchy5": (_branchy5, ())}


class UnfusedStep:
    """One forward + backward of `op` over fixed device tensors; `run()` returns (outputs, grads)."""

    def __init__(self, op, args, adjoints):
        if op not in FUNCTIONS:
            raise KeyError(f"no unfused baseline for {op}")
        self.fn, nondiff = FUNCTIONS[op]
        self.args = [a.detach().clone().requires_grad_(k not in nondiff) for k, a in enumerate(args)]
        self.leaves = [a for a in self.args if a.requires_grad]
        self.adjoints = list(adjoints)

    def run(self):
        outs = self.fn(*self.args)
        grads = torch.autograd.grad(outs, self.leaves, self.adjoints, allow_unused=True)
        return outs, [g if g is not None else torch.zeros_like(a) for g, a in zip(grads, self.leaves)]


class UnfusedPrimitives:
    """One forward + reverse pass of `op` on the library's per-primitive kernels over fixed device
    tensors (2-D, contiguous); `run()` enqueues it and returns (outputs, gradients, kernels launched)."""

    def __init__(self, op, args, adjoints):
        from . import binding as B
        self.B = B
        self.op_id = B.bcast_op_lookup(op)
        self.args = [a.contiguous() for a in args]
        self.adjoints = [a.contiguous() for a in adjoints]
        rows, cols = self.adjoints[0].shape
        n_out = B.bcast_op_info(self.op_id)[1]
        self.outs = [torch.empty_like(self.adjoints[0]) for _ in range(n_out)]
        self.grads = [torch.empty_like(self.args[j]) for j in B.diff_arg_indices(self.op_id)]
        nbytes = B.bcast_unfused_workspace(self.op_id, self.adjoints[0], rows, cols)
        if nbytes == 0:
            raise KeyError(f"no unfused program for {op}")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.adjoints[0].device)

    def run(self, stream=None):
        n = self.B.bcast_unfused_step(self.op_id, self.args, self.outs, self.adjoints, self.grads, self.workspace, stream)
        return self.outs, self.grads, n
