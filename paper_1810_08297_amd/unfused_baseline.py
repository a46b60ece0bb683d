"""Unfused reverse-mode comparison point (stands in for the paper's per-primitive graph
baseline, Sec. 3.2.1 / 3.4): the same scalar functions written as one library kernel per
primitive, every branch computed for every element and chosen with a select, differentiated by
plain reverse mode (torch.autograd).  NOT part of the product path: `bench.py --unfused-baseline`
times it next to the fused kernels, and one GPU test checks that it computes the same function.
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
