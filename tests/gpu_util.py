"""Helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle on
the same host arrays, compare element by element."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_1810_08297_amd as P

# tolerances: pass iff |gpu - oracle| <= max(rtol * |oracle|, atol)
TOL = {np.dtype(np.float32): (1e-5, 1e-6), np.dtype(np.float64): (1e-12, 1e-13)}


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_close(got, want, what, rtol=None, atol=None):
    want = np.asarray(want)
    got = np.asarray(got)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if rtol is None:
        rtol, atol = TOL[want.dtype]
    g, w = got.astype(np.float64), want.astype(np.float64)
    err = np.abs(g - w)
    tol = np.maximum(rtol * np.abs(w), atol)
    bad = ~(err <= tol)
    if bad.any():
        k = np.unravel_index(np.argmax(np.where(bad, err / tol, 0)), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at {k}: "
                             f"gpu {g[k]!r} oracle {w[k]!r} err {err[k]:.3e} tol {tol[k]:.3e}")


def gpu_forward(op, args_dev, want_branch=True, partial_mask=None, options=None):
    """Allocate buffers, run the forward kernel.  partial_mask[k] False -> plane k not stored."""
    fb = P.alloc_forward(op, args_dev, want_branch=want_branch, options=options)
    if partial_mask is not None:
        fb.partials = [p if keep else None for p, keep in zip(fb.partials, partial_mask)]
    fb.run(args_dev)
    return fb


def gpu_backward(adj_dev, partials_dev, grad_shapes, options=None):
    bb = P.alloc_backward(adj_dev, partials_dev, grad_shapes, options=options)
    bb.run(adj_dev, partials_dev)
    return bb


def full_rank(a, nd):
    """numpy view of `a` with trailing size-1 dims appended (missing dims are trailing)."""
    return a.reshape(a.shape + (1,) * (nd - a.ndim))


def check_op(op, args_np, adj_np, *, threads=8, view=None, what="", recompute=True, options=None):
    """Forward + backward parity of one op on one set of host arrays.

    `view(dev_tensor, k)` may re-lay out argument k on the device (strides, transposes)
    without changing its values.  `options`: the bcast_dual_options of every call.  Returns the
    GPU buffers for extra checks.
    """
    dt = args_np[0].dtype
    nd = max(a.ndim for a in args_np)
    args_full = [full_rank(a, nd) for a in args_np]
    o_out, o_parts, o_br = oracle.forward(op, args_full, threads=threads)
    args_dev = [to_dev(a) for a in args_np]
    if view is not None:
        args_dev = [view(t, k) for k, t in enumerate(args_dev)]
    fb = gpu_forward(op, args_dev, options=options)
    torch.cuda.synchronize()
    assert np.array_equal(fb.branch.cpu().numpy(), o_br), f"{what}{op}: branch ids differ"
    for i, (g, w) in enumerate(zip(fb.outs, o_out)):
        check_close(g.cpu().numpy(), w, f"{what}{op} output {i}")
    for k, (g, w) in enumerate(zip(fb.partials, o_parts)):
        check_close(g.cpu().numpy(), w, f"{what}{op} partial plane {k}")
    # backward: the oracle is fed the very planes the GPU backward consumes
    didx = oracle.diff_arg_indices(op, len(args_np))
    gshapes = [args_np[j].shape for j in didx]
    adj_dev = [to_dev(a) for a in adj_np]
    bb = gpu_backward(adj_dev, fb.partials, gshapes, options=options)
    torch.cuda.synchronize()
    gpu_planes = [p.cpu().numpy() for p in fb.partials]
    want = oracle.backward(adj_np, gpu_planes, [full_rank(args_np[j], nd).shape for j in didx], threads=threads)
    for k, (g, w) in enumerate(zip(bb.grads, want)):
        check_close(g.cpu().numpy().reshape(w.shape), w, f"{what}{op} gradient of argument {didx[k]}")
    # the recompute-in-reverse entry point must give the same gradients without any planes
    if recompute:
        try:
            rb = P.alloc_recompute(fb.op_id, args_dev, adj_dev, gshapes, options=options)
            P.bcast_dual_backward_recompute(fb.op_id, args_dev, adj_dev, rb.grads, rb.workspace, options=options)
        except P.BcastError as e:
            assert e.status == -12, e  # only "unsupported layout/op" is an acceptable refusal
            assert recompute != "required", f"{what}{op}: recompute refused"
        else:
            torch.cuda.synchronize()
            for k, (g, w) in enumerate(zip(rb.grads, want)):
                check_close(g.cpu().numpy().reshape(w.shape), w, f"{what}{op} recomputed gradient of argument {didx[k]}")
    return fb, bb
