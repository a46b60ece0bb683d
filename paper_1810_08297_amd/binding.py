"""Thin ctypes binding of libbcast_dual.so -- argument marshalling only.

Function names mirror the C ABI (include/bcast_dual.h).  Tensors are torch tensors
on the GPU (PyTorch supplies device memory and streams, nothing else); every step
of the method runs inside the library's kernels.  There is no CPU fallback: a
missing library raises at import of the first call.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbcast_dual.so")

MAX_DIMS = 4
MAX_ARGS = 20
MAX_OUTS = 4
MAX_PLANES = 40
F32, F64 = 0, 1


class BcastTensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("ndim", ctypes.c_int32),
                ("shape", ctypes.c_int64 * MAX_DIMS), ("stride", ctypes.c_int64 * MAX_DIMS)]


class PlanInfo(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("vec", ctypes.c_int32), ("ndim", ctypes.c_int32),
                ("shape", ctypes.c_int64 * MAX_DIMS), ("tx", ctypes.c_int32), ("ty", ctypes.c_int32),
                ("rows_per_block", ctypes.c_int32), ("grid_x", ctypes.c_int64), ("grid_y", ctypes.c_int64),
                ("n_launches", ctypes.c_int32), ("n_second_pass", ctypes.c_int32), ("specialized", ctypes.c_int32),
                ("ragged", ctypes.c_int32), ("uniform_stride", ctypes.c_int32), ("nontemporal_tiles", ctypes.c_int64)]

    def as_dict(self):
        d = {k: getattr(self, k) for k, _ in self._fields_ if k != "shape"}
        d["shape"] = list(self.shape)[: self.ndim]
        return d


class Options(ctypes.Structure):
    """bcast_dual_options: per-call launch-shape overrides and the event pair that times one
    launch.  ``Options()`` holds the library's defaults; keyword arguments change fields."""
    _fields_ = [("struct_size", ctypes.c_uint32), ("bwd_row_steps", ctypes.c_int32),
                ("nontemporal_stores", ctypes.c_int32), ("force_generic", ctypes.c_int32),
                ("max_vector_bytes", ctypes.c_int32), ("runtime_table", ctypes.c_int32),
                ("reverse_tiles", ctypes.c_int32), ("interleave_rows", ctypes.c_int32),
                ("xcd_order", ctypes.c_int32), ("col_chunks", ctypes.c_int32), ("fwd_lds_kib", ctypes.c_int32),
                ("bwd_lds_kib", ctypes.c_int32), ("narrow_tiles", ctypes.c_int32), ("ragged_rows", ctypes.c_int32),
                ("probe_nt_loads", ctypes.c_int32), ("probe_lds_kib", ctypes.c_int32), ("fwd_keep_mib", ctypes.c_int32),
                ("bwd_nt_min_mib", ctypes.c_int32), ("start_event", ctypes.c_void_p), ("stop_event", ctypes.c_void_p)]

    def __init__(self, **fields):
        super().__init__()
        lib().bcast_dual_options_default(ctypes.byref(self))
        names = {k for k, _ in self._fields_}
        for k, v in fields.items():
            if k not in names:
                raise TypeError(f"bcast_dual_options has no field {k!r}")
            setattr(self, k, v)

    def replace(self, **fields):
        """A copy with some fields changed."""
        o = Options()
        ctypes.memmove(ctypes.byref(o), ctypes.byref(self), ctypes.sizeof(Options))
        for k, v in fields.items():
            setattr(o, k, v)
        return o


def _opt(options):
    """NULL (the library's defaults) or a pointer to the caller's struct."""
    return None if options is None else ctypes.byref(options)


class BcastError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None

EXPORTS = ("bcast_op_lookup", "bcast_op_count", "bcast_op_name", "bcast_op_info", "bcast_dual_forward",
           "bcast_dual_forward_plan", "bcast_dual_backward_workspace", "bcast_dual_backward",
           "bcast_dual_backward_plan", "bcast_dual_backward_noalloc", "bcast_status_string", "bcast_dual_options_default",
           "bcast_dual_stream_probe", "bcast_dual_slab_layout", "bcast_op_plane_alias",
           "bcast_unfused_workspace", "bcast_unfused_step",
           "bcast_dual_backward_recompute", "bcast_dual_backward_recompute_workspace",
           "bcast_dual_backward_recompute_plan")


def lib():
    """Load the library built in-tree; building is a separate, explicit step."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1810_08297_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        # The library must bind to the HIP runtime that the caller's tensors and streams belong to.
        # PyTorch ships its own copy: importing it first makes that copy the one already loaded
        # when the library's dependency on libamdhip64 is resolved (loaded the other way round,
        # the library gets the system's copy and its launches fail with "no device detected").
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        # Full prototypes: ctypes then refuses a call with the wrong number of arguments instead of
        # handing the library whatever the registers hold.
        i32, i64, cint, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        T, O, PI = ctypes.POINTER(BcastTensor), ctypes.POINTER(Options), ctypes.POINTER(PlanInfo)
        proto = {
            "bcast_op_lookup": (cint, [ctypes.c_char_p, ctypes.POINTER(i32)]),
            "bcast_op_count": (cint, []),
            "bcast_op_name": (ctypes.c_char_p, [i32]),
            "bcast_op_info": (cint, [i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_uint32),
                                     ctypes.POINTER(i32)]),
            "bcast_op_plane_alias": (cint, [i32, ctypes.POINTER(i32)]),
            "bcast_dual_options_default": (None, [O]),
            "bcast_dual_forward": (cint, [i32, cint, i32, T, i32, T, T, vp, vp, O]),
            "bcast_dual_forward_plan": (cint, [i32, cint, i32, T, i32, T, T, vp, PI, O]),
            "bcast_dual_backward_workspace": (sz, [cint, i32, T, T, i32, T, O]),
            "bcast_dual_backward": (cint, [cint, i32, T, T, i32, T, vp, sz, vp, O]),
            "bcast_dual_backward_plan": (cint, [cint, i32, T, T, i32, T, PI, O]),
            "bcast_dual_backward_noalloc": (cint, [cint, i32, T, T, i32, T, vp, O]),
            "bcast_dual_backward_recompute_workspace": (sz, [i32, cint, i32, T, i32, T, i32, T, O]),
            "bcast_dual_backward_recompute": (cint, [i32, cint, i32, T, i32, T, i32, T, vp, sz, vp, O]),
            "bcast_dual_backward_recompute_plan": (cint, [i32, cint, i32, T, i32, T, i32, T, PI, O]),
            "bcast_status_string": (ctypes.c_char_p, [cint]),
            "bcast_dual_slab_layout": (sz, [sz, i32, ctypes.POINTER(sz)]),
            "bcast_dual_stream_probe": (cint, [i32, ctypes.POINTER(vp), ctypes.POINTER(i64), i32, ctypes.POINTER(vp),
                                               ctypes.POINTER(i64), i64, vp, O]),
            "bcast_unfused_workspace": (sz, [i32, cint, i64, i64]),
            "bcast_unfused_step": (cint, [i32, cint, i64, i64, i32, ctypes.POINTER(vp), ctypes.POINTER(i32), i32, ctypes.POINTER(vp),
                                          ctypes.POINTER(vp), i32, ctypes.POINTER(vp), vp, sz, vp, ctypes.POINTER(i32)]),
        }
        assert set(proto) == set(EXPORTS)
        for name, (res, argt) in proto.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, argt
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().bcast_status_string(ctypes.c_int(status)).decode()


def _check(rc, where):
    if rc != 0:
        raise BcastError(rc, where)


# ---- op table ------------------------------------------------------------------------------
def bcast_op_lookup(name: str) -> int:
    op = ctypes.c_int32()
    _check(lib().bcast_op_lookup(name.encode(), ctypes.byref(op)), f"bcast_op_lookup({name!r})")
    return op.value


def bcast_op_count() -> int:
    return lib().bcast_op_count()


def bcast_op_name(op_id: int) -> Optional[str]:
    s = lib().bcast_op_name(ctypes.c_int32(op_id))
    return None if s is None else s.decode()


def bcast_op_info(op_id: int):
    """(n_args, n_outputs, nondiff_mask, n_branches)"""
    a, m, nb = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    mask = ctypes.c_uint32()
    _check(lib().bcast_op_info(ctypes.c_int32(op_id), ctypes.byref(a), ctypes.byref(m), ctypes.byref(mask),
                               ctypes.byref(nb)), "bcast_op_info")
    return a.value, m.value, mask.value, nb.value


def bcast_op_plane_alias(op_id: int):
    """alias[k] per plane: k = own content, j < k = identical to plane j, -1 = always zero."""
    n, m, mask, _ = bcast_op_info(op_id)
    cnt = m * (n - bin(mask).count("1"))
    arr = (ctypes.c_int32 * cnt)()
    _check(lib().bcast_op_plane_alias(ctypes.c_int32(op_id), arr), "bcast_op_plane_alias")
    return [int(x) for x in arr]


def diff_arg_indices(op_id: int):
    n, _, mask, _ = bcast_op_info(op_id)
    return [j for j in range(n) if not (mask >> j) & 1]


# ---- marshalling -----------------------------------------------------------------------------
def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.float64:
        return F64
    raise TypeError(f"unsupported dtype {t.dtype}")


def as_view(t) -> BcastTensor:
    """torch tensor (or None = absent) -> bcast_tensor; strides are already in elements."""
    v = BcastTensor()
    if t is None:
        v.data, v.ndim = None, 0
        return v
    if t.dim() > MAX_DIMS:
        raise BcastError(-4, "as_view")
    v.data = t.data_ptr()
    v.ndim = t.dim()
    for d in range(t.dim()):
        v.shape[d] = t.shape[d]
        v.stride[d] = t.stride(d)
    return v


def raw_view(ptr, shape, stride) -> BcastTensor:
    v = BcastTensor()
    v.data, v.ndim = ptr, len(shape)
    for d in range(len(shape)):
        v.shape[d], v.stride[d] = shape[d], stride[d]
    return v


def _views(ts: Sequence, like=None):
    arr = (BcastTensor * max(1, len(ts)))()
    for k, t in enumerate(ts):
        arr[k] = t if isinstance(t, BcastTensor) else as_view(t)
        if t is None and like is not None:  # an absent plane keeps the common shape
            arr[k].ndim = like.ndim
            for d in range(like.ndim):
                arr[k].shape[d] = like.shape[d]
    return arr


def _on_device(*groups):
    """Launching calls hand these addresses to kernels: every tensor must live in device memory
    (a host pointer would be a memory fault on the GPU, not an error code).  The plan and
    workspace queries launch nothing and take any addresses."""
    for ts in groups:
        for t in ts or ():
            if t is not None and not isinstance(t, BcastTensor) and not t.is_cuda and t.numel() > 0:
                raise ValueError("bcast_dual: tensors of a launching call must be device tensors, got one on " + str(t.device))


def _stream_ptr(stream):
    if isinstance(stream, ctypes.c_void_p):
        return stream
    if isinstance(stream, int):  # a raw hipStream_t (0 = the default stream)
        return ctypes.c_void_p(stream)
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


# ---- forward ----------------------------------------------------------------------------------
def bcast_dual_forward(op_id: int, args: Sequence, outs: Sequence, partials: Optional[Sequence],
                       branch_id=None, stream=None, options: Optional[Options] = None) -> None:
    """Enqueue the dual-number forward kernel.  All buffers are caller-allocated."""
    _on_device(args, outs, partials, [branch_id])
    dt = _dtype_code(outs[0])
    a = _views(args)
    o = _views(outs)
    p = _views(partials, o[0]) if partials is not None else None
    _check(lib().bcast_dual_forward(
        ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(args)), a, ctypes.c_int32(len(outs)), o,
        p, ctypes.c_void_p(branch_id.data_ptr() if branch_id is not None else None), _stream_ptr(stream),
        _opt(options)), "bcast_dual_forward")


def bcast_dual_forward_plan(op_id: int, args, outs, partials, branch_id=None, options: Optional[Options] = None) -> dict:
    dt = _dtype_code(outs[0])
    a, o = _views(args), _views(outs)
    p = _views(partials, o[0]) if partials is not None else None
    info = PlanInfo()
    _check(lib().bcast_dual_forward_plan(
        ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(args)), a, ctypes.c_int32(len(outs)), o,
        p, ctypes.c_void_p(branch_id.data_ptr() if branch_id is not None else None), ctypes.byref(info),
        _opt(options)), "bcast_dual_forward_plan")
    return info.as_dict()


# ---- backward ---------------------------------------------------------------------------------
def bcast_dual_backward_workspace(adjoints, partials, grads, options: Optional[Options] = None) -> int:
    dt = _dtype_code(adjoints[0])
    a = _views(adjoints)
    return int(lib().bcast_dual_backward_workspace(
        ctypes.c_int(dt), ctypes.c_int32(len(adjoints)), a, _views(partials, a[0]),
        ctypes.c_int32(len(grads)), _views(grads), _opt(options)))


def bcast_dual_backward(adjoints, partials, grads, workspace=None, stream=None,
                        options: Optional[Options] = None) -> None:
    """Enqueue adjoint x partial with the broadcast-dim reductions.  ``workspace`` is a
    uint8 device tensor of at least bcast_dual_backward_workspace(...) bytes (or None)."""
    _on_device(adjoints, partials, grads, [workspace])
    dt = _dtype_code(adjoints[0])
    a = _views(adjoints)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().bcast_dual_backward(
        ctypes.c_int(dt), ctypes.c_int32(len(adjoints)), a, _views(partials, a[0]),
        ctypes.c_int32(len(grads)), _views(grads), ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes),
        _stream_ptr(stream), _opt(options)), "bcast_dual_backward")


NOALLOC_SCRATCH_BYTES = 16 << 20  # BCAST_NOALLOC_SCRATCH_BYTES


def bcast_dual_backward_noalloc(adjoints, partials, grads, stream=None, options: Optional[Options] = None) -> None:
    """bcast_dual_backward without a workspace argument: the second pass's scratch memory is the
    library's own static per-GPU array (for callers that cannot allocate)."""
    _on_device(adjoints, partials, grads)
    dt = _dtype_code(adjoints[0])
    a = _views(adjoints)
    _check(lib().bcast_dual_backward_noalloc(
        ctypes.c_int(dt), ctypes.c_int32(len(adjoints)), a, _views(partials, a[0]),
        ctypes.c_int32(len(grads)), _views(grads), _stream_ptr(stream), _opt(options)), "bcast_dual_backward_noalloc")


def bcast_dual_backward_plan(adjoints, partials, grads, options: Optional[Options] = None) -> dict:
    dt = _dtype_code(adjoints[0])
    a = _views(adjoints)
    info = PlanInfo()
    _check(lib().bcast_dual_backward_plan(
        ctypes.c_int(dt), ctypes.c_int32(len(adjoints)), a, _views(partials, a[0]),
        ctypes.c_int32(len(grads)), _views(grads), ctypes.byref(info), _opt(options)), "bcast_dual_backward_plan")
    return info.as_dict()


# ---- misc -------------------------------------------------------------------------------------
def bcast_dual_stream_probe(in_ptrs, in_strides, out_ptrs, out_strides, n_chunks, stream=None,
                            options: Optional[Options] = None) -> None:
    """in_ptrs/out_ptrs: device addresses (ints); strides in floats per 4 KiB chunk."""
    def arr(ctype, vals):
        return (ctype * max(1, len(vals)))(*vals)
    _check(lib().bcast_dual_stream_probe(
        ctypes.c_int32(len(in_ptrs)), arr(ctypes.c_void_p, in_ptrs), arr(ctypes.c_int64, in_strides),
        ctypes.c_int32(len(out_ptrs)), arr(ctypes.c_void_p, out_ptrs), arr(ctypes.c_int64, out_strides),
        ctypes.c_int64(n_chunks), _stream_ptr(stream), _opt(options)), "bcast_dual_stream_probe")


def bcast_dual_slab_layout(plane_bytes: int, n_planes: int):
    """(total_bytes, [offset of plane k]) of the staggered slab layout."""
    offs = (ctypes.c_size_t * max(1, n_planes))()
    total = lib().bcast_dual_slab_layout(ctypes.c_size_t(plane_bytes), ctypes.c_int32(n_planes), offs)
    return int(total), [int(offs[k]) for k in range(n_planes)]


class PreparedForward:
    """A forward call whose argument block is marshalled once; ``launch`` only enqueues.
    The tensors must stay alive and keep their addresses between launches."""

    def __init__(self, op_id, args, outs, partials, branch_id=None, options: Optional[Options] = None):
        _on_device(args, outs, partials, [branch_id])
        self._keep = (args, outs, partials, branch_id, options)
        self._opt = _opt(options)
        self._op = ctypes.c_int32(op_id)
        self._dt = ctypes.c_int(_dtype_code(outs[0]))
        self._na, self._a = ctypes.c_int32(len(args)), _views(args)
        self._no, self._o = ctypes.c_int32(len(outs)), _views(outs)
        self._p = _views(partials, self._o[0]) if partials is not None else None
        self._b = ctypes.c_void_p(branch_id.data_ptr() if branch_id is not None else None)
        self._fn = lib().bcast_dual_forward

    def launch(self, stream=None, options: Optional[Options] = None):
        """``options`` here replaces the ones given at construction for this launch (a timed one, say)."""
        _check(self._fn(self._op, self._dt, self._na, self._a, self._no, self._o, self._p, self._b,
                        _stream_ptr(stream), self._opt if options is None else ctypes.byref(options)), "bcast_dual_forward")


class PreparedBackward:
    """A backward call whose argument block is marshalled once (see PreparedForward)."""

    def __init__(self, adjoints, partials, grads, workspace=None, options: Optional[Options] = None):
        _on_device(adjoints, partials, grads, [workspace])
        self._keep = (adjoints, partials, grads, workspace, options)
        self._opt = _opt(options)
        self._dt = ctypes.c_int(_dtype_code(adjoints[0]))
        self._no, self._a = ctypes.c_int32(len(adjoints)), _views(adjoints)
        self._p = _views(partials, self._a[0])
        self._ng, self._g = ctypes.c_int32(len(grads)), _views(grads)
        self._ws = ctypes.c_void_p(workspace.data_ptr() if workspace is not None else None)
        self._wsb = ctypes.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0)
        self._fn = lib().bcast_dual_backward

    def launch(self, stream=None, options: Optional[Options] = None):
        _check(self._fn(self._dt, self._no, self._a, self._p, self._ng, self._g, self._ws, self._wsb,
                        _stream_ptr(stream), self._opt if options is None else ctypes.byref(options)), "bcast_dual_backward")


def bcast_dual_backward_recompute_workspace(op_id, args, adjoints, grads, options: Optional[Options] = None) -> int:
    dt = _dtype_code(adjoints[0])
    return int(lib().bcast_dual_backward_recompute_workspace(
        ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(args)), _views(args),
        ctypes.c_int32(len(adjoints)), _views(adjoints), ctypes.c_int32(len(grads)), _views(grads), _opt(options)))


def bcast_dual_backward_recompute_plan(op_id, args, adjoints, grads, options: Optional[Options] = None) -> dict:
    dt = _dtype_code(adjoints[0])
    info = PlanInfo()
    _check(lib().bcast_dual_backward_recompute_plan(
        ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(args)), _views(args),
        ctypes.c_int32(len(adjoints)), _views(adjoints), ctypes.c_int32(len(grads)), _views(grads),
        ctypes.byref(info), _opt(options)), "bcast_dual_backward_recompute_plan")
    return info.as_dict()


def bcast_dual_backward_recompute(op_id, args, adjoints, grads, workspace=None, stream=None,
                                  options: Optional[Options] = None) -> None:
    """Gradients straight from arguments and adjoints: the dual numbers are evaluated again."""
    _on_device(args, adjoints, grads, [workspace])
    dt = _dtype_code(adjoints[0])
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().bcast_dual_backward_recompute(
        ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(args)), _views(args),
        ctypes.c_int32(len(adjoints)), _views(adjoints), ctypes.c_int32(len(grads)), _views(grads),
        ctypes.c_void_p(ws_ptr), ctypes.c_size_t(ws_bytes), _stream_ptr(stream), _opt(options)),
        "bcast_dual_backward_recompute")


class PreparedRecompute:
    """A recompute-backward call marshalled once (see PreparedForward)."""

    def __init__(self, op_id, args, adjoints, grads, workspace=None, options: Optional[Options] = None):
        _on_device(args, adjoints, grads, [workspace])
        self._keep = (args, adjoints, grads, workspace, options)
        self._opt = _opt(options)
        self._op = ctypes.c_int32(op_id)
        self._dt = ctypes.c_int(_dtype_code(adjoints[0]))
        self._na, self._a = ctypes.c_int32(len(args)), _views(args)
        self._no, self._o = ctypes.c_int32(len(adjoints)), _views(adjoints)
        self._ng, self._g = ctypes.c_int32(len(grads)), _views(grads)
        self._ws = ctypes.c_void_p(workspace.data_ptr() if workspace is not None else None)
        self._wsb = ctypes.c_size_t(workspace.numel() * workspace.element_size() if workspace is not None else 0)
        self._fn = lib().bcast_dual_backward_recompute

    def launch(self, stream=None, options: Optional[Options] = None):
        _check(self._fn(self._op, self._dt, self._na, self._a, self._no, self._o, self._ng, self._g, self._ws,
                        self._wsb, _stream_ptr(stream), self._opt if options is None else ctypes.byref(options)),
               "bcast_dual_backward_recompute")


# ---- unfused comparison (one kernel per primitive, reverse mode) ------------------------------
UNFUSED_FULL, UNFUSED_ROW_VECTOR, UNFUSED_COL_VECTOR, UNFUSED_SCALAR = 0, 1, 2, 3


def _unfused_kind(t, rows, cols):
    shape = tuple(t.shape)
    if shape == (rows, cols):
        return UNFUSED_FULL
    if shape == (1, cols):
        return UNFUSED_ROW_VECTOR
    if shape == (rows, 1):
        return UNFUSED_COL_VECTOR
    if shape == (1, 1):
        return UNFUSED_SCALAR
    raise ValueError(f"bcast_unfused_step: an argument of shape {shape} in a problem of {rows} x {cols}")


def bcast_unfused_workspace(op_id: int, dtype_like, rows: int, cols: int) -> int:
    return int(lib().bcast_unfused_workspace(ctypes.c_int32(op_id), ctypes.c_int(_dtype_code(dtype_like)),
                                             ctypes.c_int64(rows), ctypes.c_int64(cols)))


def bcast_unfused_step(op_id: int, args, outs, adjoints, grads, workspace, stream=None) -> int:
    """Enqueue the per-primitive forward + reverse-mode chain; returns the number of kernels launched.
    All tensors contiguous 2-D device tensors; `outs`, `adjoints` full-shape, `grads` in their argument's shape."""
    _on_device(args, outs, adjoints, grads, [workspace])
    rows, cols = outs[0].shape
    for t in list(args) + list(outs) + list(adjoints) + list(grads):
        if not t.is_contiguous():
            raise ValueError("bcast_unfused_step takes contiguous tensors")
    def ptrs(ts):
        return (ctypes.c_void_p * max(1, len(ts)))(*[t.data_ptr() for t in ts])
    kinds = (ctypes.c_int32 * len(args))(*[_unfused_kind(t, rows, cols) for t in args])
    n = ctypes.c_int32()
    _check(lib().bcast_unfused_step(
        ctypes.c_int32(op_id), ctypes.c_int(_dtype_code(outs[0])), ctypes.c_int64(rows), ctypes.c_int64(cols),
        ctypes.c_int32(len(args)), ptrs(args), kinds, ctypes.c_int32(len(outs)), ptrs(outs), ptrs(adjoints),
        ctypes.c_int32(len(grads)), ptrs(grads), ctypes.c_void_p(workspace.data_ptr()),
        ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream_ptr(stream), ctypes.byref(n)), "bcast_unfused_step")
    return n.value
