"""CPU oracle (TEST INFRASTRUCTURE ONLY) -- ctypes front end of bcast_oracle.c.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It imports nothing from the HIP path.  Arrays are NumPy, contiguous,
row major, all at the same (full) rank with explicit size-1 broadcast dims.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bcast_oracle.c")
_LIB = os.path.join(_HERE, "libbcast_oracle.so")

GCC_FLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fexcess-precision=standard",
             "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FP contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *GCC_FLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_op_info.restype = ctypes.c_int
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_backward.restype = ctypes.c_int
        _lib = lib
    return _lib


def op_info(name: str):
    """(n_args, n_out, nondiff_mask); n_args == 0 means any arity."""
    n, m, mask = ctypes.c_int(), ctypes.c_int(), ctypes.c_uint32()
    rc = _load().oracle_op_info(name.encode(), ctypes.byref(n), ctypes.byref(m), ctypes.byref(mask))
    if rc:
        raise KeyError(name)
    return n.value, m.value, mask.value


def _ptr_array(arrs):
    P = (ctypes.c_void_p * len(arrs))()
    for k, a in enumerate(arrs):
        P[k] = None if a is None else a.ctypes.data
    return P


def _i64(vals):
    return (ctypes.c_int64 * len(vals))(*[int(v) for v in vals])


def forward(op: str, args, *, threads: int = 1, want_branch: bool = True):
    """Evaluate b.(X1..XN) and the diagonal Jacobian planes.

    Returns (outs[M], partials[M*N_d] in order [i*N_d + jd], branch uint8 or None).
    """
    args = [np.ascontiguousarray(a) for a in args]
    dt = args[0].dtype
    assert dt in (np.float32, np.float64) and all(a.dtype == dt for a in args)
    nd = args[0].ndim
    assert nd >= 1 and all(a.ndim == nd for a in args), "pass full-rank arrays"
    out_shape = tuple(max(a.shape[d] for a in args) for d in range(nd))
    n_args, M, mask = op_info(op)
    N = len(args)
    Nd = sum(1 for j in range(N) if not (mask >> j) & 1)
    outs = [np.empty(out_shape, dt) for _ in range(M)]
    parts = [np.empty(out_shape, dt) for _ in range(M * Nd)]
    branch = np.empty(out_shape, np.uint8) if want_branch else None
    shapes = [s for a in args for s in a.shape]
    rc = _load().oracle_forward(
        op.encode(), ctypes.c_int(dt == np.float64), ctypes.c_int(nd), _i64(out_shape),
        ctypes.c_int(N), _ptr_array(args), _i64(shapes), _ptr_array(outs), _ptr_array(parts),
        ctypes.c_void_p(branch.ctypes.data if want_branch else None), ctypes.c_int(threads))
    if rc:
        raise ValueError(f"oracle_forward({op}) failed with {rc}")
    return outs, parts, branch


def backward(adjoints, partials, grad_shapes, *, threads: int = 1):
    """grad_j = sum over j's expanded dims of sum_i adj_i * P_ij (Table 1).

    ``partials`` has M*N_d entries ([i*N_d + jd]); an entry may be None (zeros).
    ``grad_shapes`` are N_d full-rank shapes.  Returns the N_d gradients.
    """
    adjoints = [np.ascontiguousarray(a) for a in adjoints]
    dt = adjoints[0].dtype
    out_shape = adjoints[0].shape
    nd = len(out_shape)
    M, Nd = len(adjoints), len(grad_shapes)
    assert len(partials) == M * Nd
    partials = [None if p is None else np.ascontiguousarray(p) for p in partials]
    assert all(p is None or (p.dtype == dt and p.shape == out_shape) for p in partials)
    assert all(a.dtype == dt and a.shape == out_shape for a in adjoints)
    grads = [np.empty(tuple(gs), dt) for gs in grad_shapes]
    rc = _load().oracle_backward(
        ctypes.c_int(dt == np.float64), ctypes.c_int(nd), _i64(out_shape), ctypes.c_int(M),
        ctypes.c_int(Nd), _ptr_array(adjoints), _ptr_array(partials),
        _i64([s for gs in grad_shapes for s in gs]), _ptr_array(grads), ctypes.c_int(threads))
    if rc:
        raise ValueError(f"oracle_backward failed with {rc}")
    return grads


def diff_arg_indices(op: str, n_args: int):
    """Indices of the differentiable arguments, in argument order."""
    _, _, mask = op_info(op)
    return [j for j in range(n_args) if not (mask >> j) & 1]
