"""A third differentiator for pinning the oracle (test infrastructure, CPU): the ops written as
whole-array library primitives, every branch computed for every element and chosen with a
select -- no scalar `if` anywhere -- and differentiated by plain reverse mode (torch.autograd)
in fp64.  It imports neither the oracle nor the HIP package.
"""
from __future__ import annotations

import torch


def hmlstm_update(f, i, o, g, c, h, z, zb, bf, bi, bo, bg):
    flush_value = torch.sigmoid(i + bi) * torch.tanh(g + bg)
    update_value = torch.sigmoid(f + bf) * c + flush_value
    flush = z == 1
    copy = (z == 0) & (zb == 0) & ~flush
    c_new = torch.where(flush, flush_value, torch.where(copy, c, update_value))
    h_new = torch.where(copy, h, torch.sigmoid(o + bo) * torch.tanh(c_new))
    return c_new, h_new


def update_c(c, f, i, g, z1, z2):
    flush_value = torch.sigmoid(i) * torch.tanh(g)
    update_value = torch.sigmoid(f) * c + flush_value
    return (torch.where(z1 == 1, flush_value, torch.where((z1 == 0) & (z2 == 0), c, update_value)),)


def tanh_xy_b(x, y, b):
    return (torch.tanh(x * y + b),)


def branchy5(a, b, r, s, t):
    return (torch.where(a + s > t, torch.exp(-a) * b + r, torch.log1p(a * a) * r - s),)


# op -> (function, indices of its control inputs)
SELECT_FORMS = {"hmlstm_update": (hmlstm_update, (6, 7)), "update_c": (update_c, (4, 5)),
                "tanh_xy_b": (tanh_xy_b, ()), "branchy5": (branchy5, ())}


def values_and_gradients(op, args, adjoints):
    """(outputs, gradients of the differentiable arguments reduced to their shapes by autograd)."""
    fn, control = SELECT_FORMS[op]
    leaves = [a.detach().clone().requires_grad_(k not in control) for k, a in enumerate(args)]
    diff = [a for a in leaves if a.requires_grad]
    outs = fn(*leaves)
    grads = torch.autograd.grad(outs, diff, list(adjoints), allow_unused=True)
    return outs, [g if g is not None else torch.zeros_like(a) for g, a in zip(grads, diff)]
