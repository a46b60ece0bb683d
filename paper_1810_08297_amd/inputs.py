"""Seeded synthetic input generators for the broadcast workloads.

This module only draws random host arrays (NumPy) in a fixed order; it holds
none of the method's arithmetic and is the one piece of code that both the
CPU oracle's tests and the HIP path's tests/bench are allowed to share.

The paper's own workload is synthetic (random 32-bit matrices and vectors,
Sec. 3.4, results paragraph), so these arrays stand in for it directly.

Every argument is returned at full rank (2-D) with explicit size-1 dims, row
major, last dim contiguous: [hidden x batch] with batch fastest.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 181008297

#: argument order of each op (matches the op table of the library and the oracle)
HMLSTM_ARGS = ("f", "i", "o", "g", "c", "h", "z", "z_below", "b_f", "b_i", "b_o", "b_g")
TANH_XY_B_ARGS = ("x", "y", "b")
BRANCHY5_ARGS = ("A", "B", "r", "s", "t")
UPDATE_C_ARGS = ("c", "f", "i", "g", "z1", "z2")


def _normal(rng, shape, dtype, scale=1.0):
    a = rng.standard_normal(shape, dtype=np.float64 if dtype == np.float64 else np.float32)
    if scale != 1.0:
        a = a * np.asarray(scale, dtype=a.dtype)
    return np.ascontiguousarray(a.astype(dtype, copy=False))


def _bernoulli(rng, shape, p, dtype):
    return np.ascontiguousarray((rng.random(shape) < p).astype(dtype))


def hmlstm_inputs(hidden, batch, *, seed, dtype=np.float32, z_per_element=False, p=0.5):
    """HM-LSTM cell-update workload.

    Gate pre-activations f,i,o,g and previous c,h are [hidden x batch] ~ N(0,1);
    z and z_below are [1 x batch] in {0,1} ~ Bernoulli(0.5) (z becomes
    [hidden x batch] ~ Bernoulli(p) when ``z_per_element``); biases are
    [hidden x 1] ~ N(0, sd=0.1).  Adjoints for c' and h' ~ N(0,1).
    Returns (args, adjoints) as lists in op-argument order.
    """
    rng = np.random.default_rng(seed)
    full = (hidden, batch)
    f, i, o, g = (_normal(rng, full, dtype) for _ in range(4))
    c, h = (_normal(rng, full, dtype) for _ in range(2))
    if z_per_element:
        z = _bernoulli(rng, full, p, dtype)
    else:
        z = _bernoulli(rng, (1, batch), 0.5, dtype)
    z_below = _bernoulli(rng, (1, batch), 0.5, dtype)
    biases = [_normal(rng, (hidden, 1), dtype, 0.1) for _ in range(4)]
    adj = [_normal(rng, full, dtype) for _ in range(2)]
    return [f, i, o, g, c, h, z, z_below] + biases, adj


def tanh_xy_b_inputs(rows, cols, *, seed, dtype=np.float32):
    """out = tanh(x*y + b): x,y [rows x cols] ~ N(0,1), b [rows x 1] ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    x = _normal(rng, (rows, cols), dtype)
    y = _normal(rng, (rows, cols), dtype)
    b = _normal(rng, (rows, 1), dtype)
    adj = [_normal(rng, (rows, cols), dtype)]
    return [x, y, b], adj


def branchy5_inputs(rows, cols, *, seed, dtype=np.float32):
    """A ~ N(0,1), B ~ U(0.1,2) full; r [1 x cols], s [rows x 1], t scalar ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    A = _normal(rng, (rows, cols), dtype)
    B = np.ascontiguousarray(rng.uniform(0.1, 2.0, (rows, cols)).astype(dtype))
    r = _normal(rng, (1, cols), dtype)
    s = _normal(rng, (rows, 1), dtype)
    t = _normal(rng, (1, 1), dtype)
    adj = [_normal(rng, (rows, cols), dtype)]
    return [A, B, r, s, t], adj


def branchy5_3d_inputs(outer, rows, cols, *, seed, dtype=np.float32, merging=False):
    """branchy5 over [outer x rows x cols] with an argument broadcast along the middle dim only:
    r [outer x 1 x cols], s [1 x rows x 1], t scalar -- a problem that keeps three dims.
    ``merging`` gives the same elements shapes that merge to two dims instead
    (r [1 x 1 x cols], s [outer x rows x 1])."""
    rng = np.random.default_rng(seed)
    full = (outer, rows, cols)
    A = _normal(rng, full, dtype)
    B = np.ascontiguousarray(rng.uniform(0.1, 2.0, full).astype(dtype))
    r = _normal(rng, (1, 1, cols) if merging else (outer, 1, cols), dtype)
    s = _normal(rng, (outer, rows, 1) if merging else (1, rows, 1), dtype)
    t = _normal(rng, (1, 1, 1), dtype)
    adj = [_normal(rng, full, dtype)]
    return [A, B, r, s, t], adj


def update_c_inputs(n, *, seed, dtype=np.float32, uniform_run=0):
    """The paper's own experiment (Sec. 3.4): c,f,i,g n x n random, z1,z2
    n-element random control vectors varying along the contiguous dim.
    ``uniform_run`` > 0 makes both control vectors constant over aligned runs
    of that many consecutive elements (the wavefront-uniform control case)."""
    rng = np.random.default_rng(seed)
    c, f, i, g = (_normal(rng, (n, n), dtype) for _ in range(4))
    if uniform_run > 0:
        nrun = (n + uniform_run - 1) // uniform_run
        z1 = np.repeat(_bernoulli(rng, (1, nrun), 0.5, dtype), uniform_run, axis=1)[:, :n]
        z2 = np.repeat(_bernoulli(rng, (1, nrun), 0.5, dtype), uniform_run, axis=1)[:, :n]
        z1, z2 = np.ascontiguousarray(z1), np.ascontiguousarray(z2)
    else:
        z1 = _bernoulli(rng, (1, n), 0.5, dtype)
        z2 = _bernoulli(rng, (1, n), 0.5, dtype)
    adj = [_normal(rng, (n, n), dtype)]
    return [c, f, i, g, z1, z2], adj


def prod_tanh_inputs(arity, rows, cols, *, seed, dtype=np.float32):
    """Arity study (Sec. 3.4.1): N full random matrices."""
    rng = np.random.default_rng(seed)
    xs = [_normal(rng, (rows, cols), dtype) for _ in range(arity)]
    adj = [_normal(rng, (rows, cols), dtype)]
    return xs, adj


#: the five benchmark configurations: index -> (op name, builder, kwargs)
P_SWEEP = (0.05, 0.5, 0.95)


def config_inputs(index, *, dtype=np.float32, p_index=1, scale=1.0):
    """Inputs for benchmark configuration ``index`` (0..4).

    seed = BASE_SEED + index (+ 1000*k for the k-th p of configuration 3).
    ``scale`` < 1 shrinks every extent (for quick tests); 1.0 is the full size.
    Returns (op_name, args, adjoints).
    """
    def sz(n):
        return max(1, int(round(n * scale)))

    if index == 0:
        a, adj = hmlstm_inputs(sz(64), sz(16), seed=BASE_SEED + 0, dtype=dtype)
        return "hmlstm_update", a, adj
    if index == 1:
        a, adj = tanh_xy_b_inputs(sz(4096), sz(4096), seed=BASE_SEED + 1, dtype=dtype)
        return "tanh_xy_b", a, adj
    if index == 2:
        a, adj = hmlstm_inputs(sz(1024), sz(256), seed=BASE_SEED + 2, dtype=dtype)
        return "hmlstm_update", a, adj
    if index == 3:
        a, adj = hmlstm_inputs(sz(4096), sz(1024), seed=BASE_SEED + 3 + 1000 * p_index,
                               dtype=dtype, z_per_element=True, p=P_SWEEP[p_index])
        return "hmlstm_update", a, adj
    if index == 4:
        a, adj = branchy5_inputs(sz(8192), sz(8192), seed=BASE_SEED + 4, dtype=dtype)
        return "branchy5", a, adj
    raise ValueError(f"no benchmark configuration {index}")
