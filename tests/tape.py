"""A brute-force scalar reverse-mode tape (test helper, CPU only).

It is the dynamically allocated trace that the method avoids on the GPU
(Sec. 2.2.4, point 2): every scalar operation appends a node; ``backward``
walks the nodes in reverse.  Used to pin the oracle: each element of an
argument is ONE leaf, so an argument that was expanded to many output elements
collects the sum over them by construction.
"""
from __future__ import annotations

import math


class Var:
    __slots__ = ("v", "parents", "adj")

    def __init__(self, v, parents=()):
        self.v = float(v)
        self.parents = parents  # tuple of (Var, local derivative)
        self.adj = 0.0
        TAPE.append(self)

    # arithmetic ---------------------------------------------------------------
    def __add__(self, o):
        o = _lift(o)
        return Var(self.v + o.v, ((self, 1.0), (o, 1.0)))

    __radd__ = __add__

    def __sub__(self, o):
        o = _lift(o)
        return Var(self.v - o.v, ((self, 1.0), (o, -1.0)))

    def __rsub__(self, o):
        return _lift(o) - self

    def __mul__(self, o):
        o = _lift(o)
        return Var(self.v * o.v, ((self, o.v), (o, self.v)))

    __rmul__ = __mul__

    def __truediv__(self, o):
        o = _lift(o)
        return Var(self.v / o.v, ((self, 1.0 / o.v), (o, -self.v / (o.v * o.v))))

    def __rtruediv__(self, o):
        return _lift(o) / self

    def __neg__(self):
        return Var(-self.v, ((self, -1.0),))


TAPE: list = []


def _lift(x):
    return x if isinstance(x, Var) else Var(x)


def reset():
    TAPE.clear()


def exp(x):
    e = math.exp(x.v)
    return Var(e, ((x, e),))


def log1p(x):
    return Var(math.log1p(x.v), ((x, 1.0 / (1.0 + x.v)),))


def tanh(x):
    t = math.tanh(x.v)
    return Var(t, ((x, 1.0 - t * t),))


def sin(x):
    return Var(math.sin(x.v), ((x, math.cos(x.v)),))


def cos(x):
    return Var(math.cos(x.v), ((x, -math.sin(x.v)),))


def sigmoid(x):
    # composed from primitives on purpose: 1 / (1 + exp(-x))
    return 1.0 / (1.0 + exp(-x))


def backward(root):
    """Accumulate d root / d node into every node's ``adj``."""
    root.adj = 1.0
    for node in reversed(TAPE):
        if node.adj != 0.0:
            for parent, d in node.parents:
                parent.adj += node.adj * d
