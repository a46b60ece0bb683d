"""CPU-only tests of the library's host side: exported symbols, op table, argument
validation (every error is reported before anything is launched) and the plan."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import paper_1810_08297_amd as P
from paper_1810_08297_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bcast_dual.h")).read()
    body = header[header.index('extern "C"'):]
    declared = set(re.findall(r"\b(bcast_[a-z0-9_]+)\s*\(", body))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_a_c_program_links(tmp_path):
    """The boundary is a C ABI: a C99 translation unit includes the header, links against the
    library and calls entry points that touch no device (op table, plan of a call)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "client.c"
    src.write_text(r"""
#include <stdio.h>
#include <string.h>
#include "bcast_dual.h"
static bcast_tensor view(void *p, long long r, long long c) {
  bcast_tensor t; memset(&t, 0, sizeof t);
  t.data = p; t.ndim = 2; t.shape[0] = r; t.shape[1] = c; t.stride[0] = c; t.stride[1] = 1;
  return t;
}
int main(void) {
  int32_t op = -1, n_args = 0, n_out = 0, n_br = 0; uint32_t mask = 0;
  bcast_tensor args[3], outs[1], parts[3];
  bcast_plan_info info;
  bcast_dual_options opt;
  char *base = (char *)0;  /* addresses are planned with, never dereferenced */
  int k;
  if (bcast_op_lookup("tanh_xy_b", &op) != BCAST_OK) return 1;
  if (bcast_op_info(op, &n_args, &n_out, &mask, &n_br) != BCAST_OK || n_args != 3 || n_out != 1) return 2;
  args[0] = view(base + (1 << 24), 512, 1024); args[1] = view(base + (2 << 24), 512, 1024);
  args[2] = view(base + (3 << 24), 512, 1);
  outs[0] = view(base + (4 << 24), 512, 1024);
  for (k = 0; k < 3; ++k) parts[k] = view(base + ((5 + k) << 24), 512, 1024);
  bcast_dual_options_default(&opt);
  if (opt.struct_size != sizeof opt) return 4;
  if (bcast_dual_forward_plan(op, BCAST_F32, 3, args, 1, outs, parts, NULL, &info, &opt) != BCAST_OK) return 3;
  if (bcast_dual_forward_plan(op, BCAST_F32, 3, args, 1, outs, parts, NULL, &info, NULL) != BCAST_OK) return 5;
  printf("%d %d %lld %lld %s\n", (int)info.path, (int)info.vec, (long long)info.shape[0], (long long)info.shape[1],
         bcast_status_string(BCAST_ERR_WORKSPACE_TOO_SMALL));
  return 0;
}
""")
    exe = tmp_path / "client"
    libdir = os.path.dirname(B.LIB_PATH)
    libname = os.path.basename(B.LIB_PATH)
    B.lib()  # the library (and the HIP runtime it needs) is loadable here
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
           "-o", str(exe), "-L", libdir, "-l:" + libname, "-Wl,-rpath," + libdir, "-Wl,--allow-shlib-undefined"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ)
    torch_lib = os.path.join(os.path.dirname(torch.__file__), "lib")
    env["LD_LIBRARY_PATH"] = os.pathsep.join([torch_lib, "/opt/rocm/lib", env.get("LD_LIBRARY_PATH", "")])
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    path, vec, rows, cols, msg = r.stdout.split(maxsplit=4)
    assert (int(path), int(vec), int(rows), int(cols)) == (1, 4, 512, 1024) and "workspace" in msg


def test_op_table():
    names = [P.bcast_op_name(k) for k in range(P.bcast_op_count())]
    for n in ("hmlstm_update", "tanh_xy_b", "branchy5", "update_c", "cos_x", "scale_xt", "pair3",
              "prod_tanh_1", "prod_tanh_18"):
        assert n in names
    assert P.bcast_op_name(-1) is None and P.bcast_op_name(10 ** 6) is None
    op = P.bcast_op_lookup("hmlstm_update")
    assert P.bcast_op_info(op) == (12, 2, (1 << 6) | (1 << 7), 3)
    assert P.diff_arg_indices(op) == [0, 1, 2, 3, 4, 5, 8, 9, 10, 11]
    assert P.bcast_op_info(P.bcast_op_lookup("branchy5")) == (5, 1, 0, 2)
    with pytest.raises(P.BcastError) as e:
        P.bcast_op_lookup("no_such_op")
    assert e.value.status == -1
    assert P.status_string(0) == "ok" and "workspace" in P.status_string(-8)


def _t(*shape, dtype=torch.float32):
    return torch.zeros(shape, dtype=dtype)


def _fwd_status(op, args, outs, parts, branch=None):
    try:
        P.bcast_dual_forward_plan(P.bcast_op_lookup(op), args, outs, parts, branch)
        return 0
    except P.BcastError as e:
        return e.status


def test_forward_validation_errors():
    x, y, b = _t(4, 6), _t(4, 6), _t(4, 1)
    out, parts = [_t(4, 6)], [_t(4, 6) for _ in range(3)]
    assert _fwd_status("tanh_xy_b", [x, y, b], out, parts) == 0
    assert _fwd_status("tanh_xy_b", [x, y], out, parts) == -2                      # argument count
    assert _fwd_status("tanh_xy_b", [x, _t(4, 5), b], out, parts) == -5           # not broadcastable
    assert _fwd_status("tanh_xy_b", [x, y, b], [_t(4, 1)], parts) == -6           # output shape
    assert _fwd_status("tanh_xy_b", [x, y, b], out, [_t(4, 6), _t(6, 4), _t(4, 6)]) == -6
    assert _fwd_status("tanh_xy_b", [x, y, b], [_t(4, 6).expand(4, 6)[:, :1].expand(4, 6)], parts) == -10
    v = B.as_view(x)
    v.ndim = 5
    assert _fwd_status("tanh_xy_b", [v, y, b], out, parts) == -4
    v = B.as_view(x)
    v.data = None
    assert _fwd_status("tanh_xy_b", [v, y, b], out, parts) == -3
    v = B.as_view(x)
    v.data = x.data_ptr() + 2
    assert _fwd_status("tanh_xy_b", [v, y, b], out, parts) == -11
    v = B.as_view(x)
    v.stride[0] = -6
    assert _fwd_status("tanh_xy_b", [v, y, b], out, parts) == -10
    # the real entry point reports the same errors and launches nothing (no GPU here)
    def real(op_id, a):  # straight through ctypes: the Python wrapper would refuse host tensors first
        return B.lib().bcast_dual_forward(ctypes.c_int32(op_id), ctypes.c_int(0), ctypes.c_int32(len(a)), B._views(a),
                                          ctypes.c_int32(1), B._views(out), B._views(parts), None, None, None)

    assert real(P.bcast_op_lookup("tanh_xy_b"), [x, y]) == -2
    assert real(999, [x, y, b]) == -1
    rc = B.lib().bcast_dual_forward(ctypes.c_int32(1), ctypes.c_int(7), ctypes.c_int32(3), B._views([x, y, b]),
                                    ctypes.c_int32(1), B._views(out), B._views(parts), None, None, None)
    assert rc == -7


def test_zero_sized_problem_is_ok_and_launches_nothing():
    x, y, b = _t(0, 6), _t(0, 6), _t(0, 1)
    info = P.bcast_dual_forward_plan(P.bcast_op_lookup("tanh_xy_b"), [x, y, b], [_t(0, 6)],
                                     [_t(0, 6) for _ in range(3)])
    assert info["path"] == 0 and info["n_launches"] == 0
    P.bcast_dual_forward(P.bcast_op_lookup("tanh_xy_b"), [x, y, b], [_t(0, 6)],
                         [_t(0, 6) for _ in range(3)], stream=0)
    P.bcast_dual_backward([_t(0, 6)], [_t(0, 6)] * 3, [_t(0, 6), _t(0, 6), _t(0, 1)], None, stream=0)


def test_forward_plan_geometry():
    op = P.bcast_op_lookup("hmlstm_update")

    def hm(H, Bt, z_full=False, dtype=torch.float32):
        full = lambda: _t(H, Bt, dtype=dtype)
        args = [full() for _ in range(6)] + [full() if z_full else _t(1, Bt, dtype=dtype), _t(1, Bt, dtype=dtype)] + \
               [_t(H, 1, dtype=dtype) for _ in range(4)]
        return args, [full(), full()], [full() for _ in range(20)]

    a, o, p = hm(4096, 1024)
    info = P.bcast_dual_forward_plan(op, a, o, p)
    assert info["path"] == 1 and info["vec"] == 4 and info["shape"] == [4096, 1024]
    assert info["tx"] == 256 and info["ty"] == 1 and info["n_launches"] == 1
    assert info["grid_x"] * info["grid_y"] * info["rows_per_block"] >= 4096
    a, o, p = hm(64, 16)
    info = P.bcast_dual_forward_plan(op, a, o, p)
    assert info["tx"] == 4 and info["ty"] == 64 and info["grid_x"] * info["grid_y"] == 1
    a, o, p = hm(64, 15)  # odd row length: unaligned vectors and a tail, or (option ragged_rows off) scalar accesses
    info = P.bcast_dual_forward_plan(op, a, o, p)
    assert info["vec"] == 4 and info["ragged"] == 1
    info = P.bcast_dual_forward_plan(op, a, o, p, options=P.Options(ragged_rows=0))
    assert info["vec"] == 1 and info["ragged"] == 0
    a, o, p = hm(64, 3)  # a row shorter than the vector
    info = P.bcast_dual_forward_plan(op, a, o, p)
    assert info["vec"] == 1 and info["ragged"] == 0
    a, o, p = hm(64, 16, dtype=torch.float64)
    assert P.bcast_dual_forward_plan(op, a, o, p)["vec"] == 2
    # everything contiguous and full-shape: the two dims merge into one
    op1 = P.bcast_op_lookup("cos_x")
    info = P.bcast_dual_forward_plan(op1, [_t(8, 32)], [_t(8, 32)], [_t(8, 32)])
    assert info["ndim"] == 1 and info["shape"] == [256]
    # column-major data is the same problem with the dims swapped
    xt = _t(32, 8).t()
    info = P.bcast_dual_forward_plan(op1, [xt], [_t(32, 8).t()], [_t(32, 8).t()])
    assert info["path"] == 1 and info["shape"] == [256]
    # a transposed input against row-major outputs needs the generic kernel
    info = P.bcast_dual_forward_plan(op1, [xt], [_t(8, 32)], [_t(8, 32)])
    assert info["path"] == 2
    # rank 4 that cannot merge
    x4 = _t(3, 5, 7, 9)[:, :4, :6, :8]
    info = P.bcast_dual_forward_plan(op1, [x4], [torch.zeros_like(x4)], [torch.zeros_like(x4)])
    assert info["path"] == 2 and info["ndim"] == 4
    # missing dims are trailing (the n-vector pairs with the first dim, Sec. 2.1.1 Eq. 1)
    op3 = P.bcast_op_lookup("pair3")
    A, alpha, a = _t(2, 3), _t(1), _t(2)
    outs, parts = [_t(2, 3), _t(2, 3)], [_t(2, 3) for _ in range(6)]
    assert P.bcast_dual_forward_plan(op3, [A, alpha, a], outs, parts)["path"] == 1
    with pytest.raises(P.BcastError):
        P.bcast_dual_forward_plan(op3, [A, alpha, _t(3)], outs, parts)


def test_backward_plan_and_workspace():
    R, C = 8192, 8192
    big = torch.empty(0)

    def fake(shape):  # shapes only: a view over no real memory, never dereferenced by the planner
        st, acc = [], 1
        for s in reversed(shape):
            st.append(acc)
            acc *= s
        return B.raw_view(4096, shape, list(reversed(st)))

    adj = [fake((R, C))]
    parts = [fake((R, C)) for _ in range(5)]
    grads = [fake((R, C)), fake((R, C)), fake((1, C)), fake((R, 1)), fake((1, 1))]
    L = B.lib()
    info = B.PlanInfo()
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                    ctypes.c_int32(5), B._views(grads), ctypes.byref(info), None)
    assert rc == 0
    d = info.as_dict()
    assert d["path"] == 1 and d["vec"] == 4 and d["n_second_pass"] == 3 and d["n_launches"] == 2
    n_ct, n_rt = d["grid_x"], d["grid_y"]
    assert n_ct == 8 and d["rows_per_block"] == 128  # two blocks per CU for the kernels that read the table at run time
    assert d["specialized"] == 0  # every plane at one address: not a layout a class-specialised kernel was built for
    distinct = [B.raw_view(4096 + (k + 1) * (1 << 30), (R, C), (C, 1)) for k in range(5)]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(distinct),
                                    ctypes.c_int32(5), B._views(grads), ctypes.byref(info), None)
    assert rc == 0 and info.specialized == 1  # config 4 runs the kernel compiled for full, full, col-sum, row-sum, all-sum
    assert info.rows_per_block == 256 and info.grid_y == 32  # ... as one block per CU
    ws = L.bcast_dual_backward_workspace(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                         ctypes.c_int32(5), B._views(grads), None)
    assert ws == 8 * (n_rt * C + R * n_ct + n_rt * n_ct)
    ws64 = L.bcast_dual_backward_workspace(ctypes.c_int(1), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                           ctypes.c_int32(5), B._views(grads), None)
    assert ws64 > ws
    # too small a workspace is refused before any launch
    rc = L.bcast_dual_backward(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                               ctypes.c_int32(5), B._views(grads), ctypes.c_void_p(4096), ctypes.c_size_t(64), None, None)
    assert rc == -8
    rc = L.bcast_dual_backward(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                               ctypes.c_int32(5), B._views(grads), None, ctypes.c_size_t(0), None, None)
    assert rc == -3
    # HM-LSTM at batch <= 1024: bias row sums finish inside the main pass
    H, Bt = 4096, 1024
    adj = [fake((H, Bt))] * 2
    parts = [fake((H, Bt))] * 20
    grads = [fake((H, Bt))] * 6 + [fake((H, 1))] * 4
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj), B._views(parts),
                                    ctypes.c_int32(10), B._views(grads), ctypes.byref(info), None)
    assert rc == 0 and info.n_launches == 1 and info.n_second_pass == 0
    parts_distinct = [B.raw_view(4096 + (k + 1) * (1 << 30), (H, Bt), (Bt, 1)) for k in range(20)]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj), B._views(parts_distinct),
                                    ctypes.c_int32(10), B._views(grads), ctypes.byref(info), None)
    assert rc == 0 and info.specialized == 1 and info.rows_per_block == 1  # config 3: class-specialised, no row loop
    assert L.bcast_dual_backward_workspace(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj), B._views(parts),
                                           ctypes.c_int32(10), B._views(grads), None) == 0
    # the same update stored [batch x hidden]: bias gradients are sums over rows; the kernel built
    # for that mix streams 22 planes per row step and runs as two blocks per CU, the lean layout
    # (12 distinct planes) as one
    adj_t = [B.raw_view(4096 + (40 + k) * (1 << 30), (Bt, H), (H, 1)) for k in range(2)]
    parts_t = [B.raw_view(4096 + (k + 1) * (1 << 30), (Bt, H), (H, 1)) for k in range(20)]
    grads_t = [fake((Bt, H))] * 6 + [fake((1, H))] * 4
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj_t), B._views(parts_t),
                                    ctypes.c_int32(10), B._views(grads_t), ctypes.byref(info), None)
    assert rc == 0 and info.specialized == 1 and info.n_second_pass == 4
    assert info.grid_x == 4 and info.rows_per_block == 8 and info.grid_y == 128
    alias = P.bcast_op_plane_alias(P.bcast_op_lookup("hmlstm_update"))
    lean_t = [None if a < 0 else parts_t[a] for a in alias]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj_t), B._views(lean_t, adj_t[0]),
                                    ctypes.c_int32(10), B._views(grads_t), ctypes.byref(info), None)
    assert rc == 0 and info.specialized == 1 and info.rows_per_block == 16 and info.grid_y == 64
    # config 1: a 4096-wide row is four column chunks; the kernel built for it takes all four in
    # one block, so the bias gradient's row sums need neither workspace nor second pass
    adj1 = [fake((4096, 4096))]
    parts1 = [B.raw_view(4096 + (k + 1) * (1 << 30), (4096, 4096), (4096, 1)) for k in range(3)]
    grads1 = [fake((4096, 4096)), fake((4096, 4096)), fake((4096, 1))]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj1), B._views(parts1),
                                    ctypes.c_int32(3), B._views(grads1), ctypes.byref(info), None)
    assert rc == 0 and info.specialized == 1 and info.n_launches == 1 and info.n_second_pass == 0 and info.grid_x == 1
    assert L.bcast_dual_backward_workspace(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj1), B._views(parts1),
                                           ctypes.c_int32(3), B._views(grads1), None) == 0
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj1), B._views(parts1),
                                    ctypes.c_int32(3), B._views(grads1), ctypes.byref(info), ctypes.byref(P.Options(col_chunks=0)))
    assert rc == 0 and info.n_launches == 2 and info.n_second_pass == 1 and info.grid_x == 4
    # gradient shape that is neither the adjoint's nor 1
    bad = grads[:9] + [fake((H, 2))]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(2), B._views(adj), B._views(parts),
                                    ctypes.c_int32(10), B._views(bad), ctypes.byref(info), None)
    assert rc == -6
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(5), B._views(adj * 3), B._views(parts),
                                    ctypes.c_int32(10), B._views(grads), ctypes.byref(info), None)
    assert rc == -2


def test_expanded_read_views_break_the_common_row_stride():
    """A plane or an adjoint that repeats one row over all rows (row stride 0, an expanded view) is a view
    with a row stride of its own: the kernels built for ONE common row stride would address it with the
    others' stride and run past its single row.  The plan must not be the uniform-stride one, whichever
    view it is (the first adjoint is the planner's sort key; any other used to slip through)."""
    R, C = 512, 1024
    slot = 1 << 30
    full = lambda k: B.raw_view(4096 + k * slot, (R, C), (C, 1))
    rowrep = lambda k: B.raw_view(4096 + k * slot, (R, C), (0, 1))
    grads3 = [full(10), full(11), B.raw_view(4096 + 12 * slot, (R, 1), (1, 1))]

    def plan(adj, parts, grads):
        info = B.PlanInfo()
        rc = B.lib().bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(len(adj)), B._views(adj), B._views(parts),
                                              ctypes.c_int32(len(grads)), B._views(grads), ctypes.byref(info), None)
        assert rc == 0
        return info.as_dict()

    def plan_recompute(op, args, adj, grads):
        info = B.PlanInfo()
        rc = B.lib().bcast_dual_backward_recompute_plan(ctypes.c_int32(op), ctypes.c_int(0), ctypes.c_int32(len(args)), B._views(args),
                                                        ctypes.c_int32(len(adj)), B._views(adj), ctypes.c_int32(len(grads)),
                                                        B._views(grads), ctypes.byref(info), None)
        assert rc == 0
        return info.as_dict()

    base = plan([full(0)], [full(1), full(2), full(3)], grads3)
    assert base["path"] == 1 and base["specialized"] == 1 and base["uniform_stride"] == 1
    for k in range(3):  # each plane in turn
        parts = [full(1), full(2), full(3)]
        parts[k] = rowrep(1 + k)
        d = plan([full(0)], parts, grads3)
        assert d["path"] == 2 or d["uniform_stride"] == 0, (k, d)
    # M = 2: a row-expanded SECOND adjoint
    grads2 = [full(10), full(11)]
    d = plan([full(0), full(5)], [full(1), full(2), full(3), full(4)], grads2)
    assert d["path"] == 1 and d["uniform_stride"] == 1
    d = plan([full(0), rowrep(5)], [full(1), full(2), full(3), full(4)], grads2)
    assert d["path"] == 2 or d["uniform_stride"] == 0, d
    # an expanded plane that starts where a full plane starts is not "the same plane stored once"
    d = plan([full(0)], [full(1), rowrep(1), full(3)], grads3)
    assert d["path"] == 2 or d["uniform_stride"] == 0, d
    # the recompute entry point streams the adjoints the same way
    op = P.bcast_op_lookup("pair3")
    args = [full(20), full(21), full(22)]
    g3 = [full(10), full(11), full(12)]
    d = plan_recompute(op, args, [full(0), full(5)], g3)
    assert d["path"] == 1 and d["uniform_stride"] == 1
    d = plan_recompute(op, args, [full(0), rowrep(5)], g3)
    assert d["uniform_stride"] == 0, d


def test_nontemporal_store_policy_by_size():
    """Which stores carry the nontemporal hint follows from how the bytes written compare with the caches: a
    forward launch that writes up to 128 MiB hints everything, up to 1 GiB nothing, beyond that all but the last
    256 MiB of its walk; a backward call hints its full-shape gradients when it reads at most 128 MiB of planes or
    writes at least 256 MiB of gradients.  Options move or switch off each rule."""
    # tanh_xy_b writes 1 + 3 planes and has 2 full-shape gradients
    def plans(R, C, **opt):
        slot = 1 << 36
        view = lambda k, shape: B.raw_view(4096 + k * slot, shape, (shape[1], 1))
        x, y, b = view(0, (R, C)), view(1, (R, C)), view(2, (R, 1))
        outs, parts = [view(3, (R, C))], [view(4 + k, (R, C)) for k in range(3)]
        grads = [view(8, (R, C)), view(9, (R, C)), view(10, (R, 1))]
        o = P.Options(**opt) if opt else None
        rc, f = _fwd_plan("tanh_xy_b", 0, [x, y, b], outs, parts, o)
        assert rc == 0
        info = B.PlanInfo()
        rc = B.lib().bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(outs), B._views(parts), ctypes.c_int32(3),
                                              B._views(grads), ctypes.byref(info), None if o is None else ctypes.byref(o))
        assert rc == 0
        return f, info.as_dict()

    f, r = plans(1024, 1024)      # 16 MiB written, 16 MiB of planes read
    assert f["nontemporal_tiles"] == f["grid_x"] * f["grid_y"] and r["nontemporal_tiles"] == r["grid_x"] * r["grid_y"] > 0
    f, r = plans(4096, 4096)      # 256 MiB written; 256 MiB of planes, 128 MiB of gradients
    assert f["nontemporal_tiles"] == 0 and r["nontemporal_tiles"] == 0
    f, r = plans(8192, 16384)     # 2 GiB written; 1 GiB of gradients
    tiles = f["grid_x"] * f["grid_y"]
    tile_bytes = 4 * f["ty"] * f["tx"] * f["vec"] * 4
    assert f["nontemporal_tiles"] == tiles - (256 << 20) // tile_bytes and r["nontemporal_tiles"] > 0
    f, r = plans(8192, 16384, nontemporal_stores=0)
    assert f["nontemporal_tiles"] == 0 and r["nontemporal_tiles"] == 0
    f, r = plans(8192, 16384, fwd_keep_mib=0, bwd_nt_min_mib=2048)
    assert f["nontemporal_tiles"] == tiles and r["nontemporal_tiles"] == 0
    f, r = plans(4096, 4096, fwd_keep_mib=64, bwd_nt_min_mib=0, col_chunks=0)  # (the kernels that take a row's four column chunks have no such form)
    assert f["nontemporal_tiles"] == f["grid_x"] * f["grid_y"] - (64 << 20) // (4 * f["ty"] * f["tx"] * f["vec"] * 4) and r["nontemporal_tiles"] > 0
    # the backward kernels that read the gradient table at run time have no such form
    f, r = plans(8192, 16384, runtime_table=1)
    assert r["specialized"] == 0 and r["nontemporal_tiles"] == 0


def test_options_defaults_ranges_and_struct_size():
    """NULL options and a default-filled struct plan alike; a field outside its range, a struct of another
    size or half an event pair are refused with BCAST_ERR_BAD_OPTION before anything else is looked at."""
    o = P.Options()
    assert o.struct_size == ctypes.sizeof(P.Options) and (o.nontemporal_stores, o.reverse_tiles, o.fwd_lds_kib) == (3, 2, -1)
    assert (o.max_vector_bytes, o.interleave_rows, o.col_chunks, o.narrow_tiles, o.ragged_rows, o.probe_nt_loads) == (16, 1, 1, 1, 1, 1)
    assert (o.bwd_row_steps, o.force_generic, o.runtime_table, o.xcd_order, o.bwd_lds_kib, o.probe_lds_kib) == (0,) * 6
    assert o.start_event is None and o.stop_event is None and (o.fwd_keep_mib, o.bwd_nt_min_mib) == (-1, -1)
    x, y, b = _t(64, 2048), _t(64, 2048), _t(64, 1)
    outs, parts = [_t(64, 2048)], [_t(64, 2048) for _ in range(3)]
    op = P.bcast_op_lookup("tanh_xy_b")
    assert P.bcast_dual_forward_plan(op, [x, y, b], outs, parts) == P.bcast_dual_forward_plan(op, [x, y, b], outs, parts, options=o)
    assert P.bcast_dual_forward_plan(op, [x, y, b], outs, parts, options=P.Options(force_generic=1))["path"] == 2
    bad = [P.Options(bwd_row_steps=513), P.Options(bwd_row_steps=-1), P.Options(nontemporal_stores=4), P.Options(max_vector_bytes=12),
           P.Options(fwd_lds_kib=65), P.Options(fwd_lds_kib=-2), P.Options(fwd_keep_mib=-2), P.Options(bwd_nt_min_mib=(1 << 20) + 1), P.Options(reverse_tiles=3), P.Options(force_generic=2), P.Options(struct_size=ctypes.sizeof(P.Options) - 8),
           P.Options(start_event=4096), P.Options(stop_event=4096)]
    for opt in bad:
        with pytest.raises(P.BcastError) as e:
            P.bcast_dual_forward_plan(op, [x, y, b], outs, parts, options=opt)
        assert e.value.status == -13
        with pytest.raises(P.BcastError) as e:
            P.bcast_dual_backward_plan(outs, parts, [x, y, b], options=opt)
        assert e.value.status == -13
        assert P.bcast_dual_backward_workspace(outs, parts, [x, y, b], options=opt) == 0
    assert "option" in P.status_string(-13)
    with pytest.raises(TypeError):
        P.Options(no_such_field=1)


def test_calls_from_two_threads_with_different_options_do_not_interfere():
    """The library keeps no state between calls: plans made concurrently from two host threads, each with
    options of its own, come out as they do alone."""
    import threading
    x, y, b = _t(300, 1100), _t(300, 1100), _t(300, 1)
    outs, parts = [_t(300, 1100)], [_t(300, 1100) for _ in range(3)]
    op = P.bcast_op_lookup("tanh_xy_b")
    opts = [P.Options(), P.Options(force_generic=1), P.Options(max_vector_bytes=4), P.Options(bwd_row_steps=5, runtime_table=1)]
    alone = [(P.bcast_dual_forward_plan(op, [x, y, b], outs, parts, options=o),
              P.bcast_dual_backward_plan(outs, parts, [x, y, b], options=o)) for o in opts]
    assert len({str(a) for a in alone}) == len(opts)  # the options do change the plan
    wrong = []

    def worker(k):
        for _ in range(300):
            got = (P.bcast_dual_forward_plan(op, [x, y, b], outs, parts, options=opts[k]),
                   P.bcast_dual_backward_plan(outs, parts, [x, y, b], options=opts[k]))
            if got != alone[k]:
                wrong.append(k)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(len(opts))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not wrong


def test_plane_alias_table_agrees_with_the_oracle():
    """Planes the op table calls identical or zero are so in the oracle, on inputs that reach
    every branch; everything else has content of its own."""
    import oracle
    rng = np.random.default_rng(3)
    R, C = 12, 16
    full, row, col, sc = (R, C), (1, C), (R, 1), (1, 1)
    cases = {
        "hmlstm_update": [full] * 6 + [row, row] + [col] * 4,
        "branchy5": [full, full, row, col, sc],
        "tanh_xy_b": [full, full, col],
        "update_c": [full] * 4 + [row, row],
    }
    for op, shp in cases.items():
        args = [rng.standard_normal(s) for s in shp]
        if op == "hmlstm_update":
            args[6] = np.array([[1, 0, 0, 1] * 4], float)
            args[7] = np.array([[0, 0, 1, 1] * 4], float)
        if op == "update_c":
            args[4] = np.array([[1, 0, 0, 1] * 4], float)
            args[5] = np.array([[0, 0, 1, 1] * 4], float)
        _, planes, br = oracle.forward(op, args)
        assert len(np.unique(br)) == {"hmlstm_update": 3, "update_c": 3, "branchy5": 2, "tanh_xy_b": 1}[op]
        alias = P.bcast_op_plane_alias(P.bcast_op_lookup(op))
        assert len(alias) == len(planes)
        for k, a in enumerate(alias):
            if a < 0:
                assert np.all(planes[k] == 0), (op, k)
            elif a != k:
                assert a < k and alias[a] == a and np.array_equal(planes[k], planes[a]), (op, k)
            else:
                assert np.any(planes[k] != 0), (op, k)
                assert all(not np.array_equal(planes[k], planes[j]) for j in range(k) if alias[j] == j), (op, k)
    assert P.bcast_op_plane_alias(P.bcast_op_lookup("hmlstm_update")).count(-1) == 3


def test_shared_plane_views_only_where_declared_identical():
    op = P.bcast_op_lookup("hmlstm_update")
    H, Bt = 8, 16
    full = lambda: _t(H, Bt)
    args = [full() for _ in range(6)] + [_t(1, Bt), _t(1, Bt)] + [_t(H, 1) for _ in range(4)]
    outs = [full(), full()]
    parts = [full() for _ in range(20)]
    parts[6] = parts[0]          # d c'/d b_f shares d c'/d f: declared identical
    P.bcast_dual_forward_plan(op, args, outs, parts)
    parts[1] = parts[0]          # d c'/d i is not
    with pytest.raises(P.BcastError) as e:
        P.bcast_dual_forward_plan(op, args, outs, parts)
    assert e.value.status == -10


def _rowmajor(ptr, shape):
    st, acc = [], 1
    for s in reversed(shape):
        st.append(acc if s > 1 else 0)
        acc *= s
    return B.raw_view(ptr, shape, list(reversed(st)))


def _fwd_plan(op_name, dt, args, outs, parts, opt=None):
    info = B.PlanInfo()
    rc = B.lib().bcast_dual_forward_plan(ctypes.c_int32(P.bcast_op_lookup(op_name)), ctypes.c_int(dt),
                                         ctypes.c_int32(len(args)), B._views(args), ctypes.c_int32(len(outs)),
                                         B._views(outs), B._views(parts), None, ctypes.byref(info),
                                         None if opt is None else ctypes.byref(opt))
    return rc, info.as_dict()


def test_alignment_and_offset_range_pick_the_access_width_and_the_kernel():
    """The planner (no memory is touched: the views point at addresses that are never
    dereferenced) narrows the vector width to what every pointer is aligned to, refuses
    pointers not aligned to the element, and keeps the tiled kernels for planes of any size as long
    as the rows of one block's row step span less than 4 GiB."""
    R, C = 512, 1024
    slot = 1 << 34  # written views must not overlap: every view gets an address range of its own

    def call(dt, shape, shifts=(0, 0), col=None, stride=None, opt=None):
        mk = (lambda k, sh=0: B.raw_view((k + 1) * slot + sh, shape, stride)) if stride else \
             (lambda k, sh=0: _rowmajor((k + 1) * slot + sh, shape))
        args = [mk(0, shifts[0]), mk(1, shifts[1]), _rowmajor(9 * slot, col or (shape[0], 1))]
        return _fwd_plan("tanh_xy_b", dt, args, [mk(2)], [mk(3), mk(4), mk(5)], opt)

    # by default a pointer or row stride off the 16-byte boundary sends the call to the kernels that
    # take unaligned vectors; with the option ragged_rows off the access narrows to what is aligned
    for ragged_on in (1, 0):
        opt = P.Options(ragged_rows=ragged_on)
        for shift, vec in ((0, 4), (8, 2), (4, 1), (12, 1)):
            rc, d = call(0, (R, C), (0, shift), opt=opt)
            assert rc == 0 and d["path"] == 1, (shift, d)
            assert (d["vec"], d["ragged"]) == ((4, int(shift != 0)) if ragged_on else (vec, 0)), (shift, d)
        rc, d = call(1, (R, C), (0, 8), opt=opt)  # fp64: 8-byte alignment allows one element per aligned access
        assert rc == 0 and (d["vec"], d["ragged"]) == ((2, 1) if ragged_on else (1, 0))
        assert call(0, (R, C), (2, 0), opt=opt)[0] == -11
        assert call(1, (R, C), (4, 0), opt=opt)[0] == -11
        # a row stride that is not a multiple of the vector width
        rc, d = call(0, (R, C), stride=(C + 2, 1), opt=opt)
        assert rc == 0 and d["path"] == 1 and (d["vec"], d["ragged"]) == ((4, 1) if ragged_on else (2, 0))
    # Planes of any size: a lane's 32-bit byte offset counts from the first row of its block's row
    # step, so only one step of rows has to span less than 4 GiB.  40000 x 30000 fp32 = 4.8 GB per plane:
    rc, d = call(0, (40000, 30000))
    assert rc == 0 and d["path"] == 1 and d["vec"] == 4 and d["ty"] == 1
    rc, d = call(1, (70000, 16384))  # 9.2 GB per plane
    assert rc == 0 and d["path"] == 1 and d["vec"] == 2
    # short rows far apart: the 256 rows of one step would span 255 * 2^23 * 4 bytes > 4 GiB
    rc, d = call(0, (4096, 512), stride=(1 << 23, 1))
    assert rc == 0 and d["path"] == 2
    rc, d = call(0, (4096, 512), stride=(1 << 21, 1))
    assert rc == 0 and d["path"] == 1 and d["ty"] == 2
    rc, d = call(0, (4096, 1024), stride=(1 << 30, 1))  # one row per step: any row stride
    assert rc == 0 and d["path"] == 1 and d["ty"] == 1
    # contiguous dims are fused only up to 2^28 elements, never into a row longer than the lanes
    # can address: 16 x 4096 x 2^15 (8 GiB fp32) becomes [2^16 x 2^15], not one dim
    mk = lambda k, shape: _rowmajor((k + 1) * slot * 4, shape)
    big = (16, 4096, 1 << 15)
    rc, d = _fwd_plan("cos_x", 0, [mk(0, big)], [mk(1, big)], [mk(2, big)])
    assert rc == 0 and d["path"] == 1 and d["shape"] == [1 << 16, 1 << 15]
    # ... and so is a long vector handed over as one dim, if a power of two divides it
    vec1 = (3 << 29,)
    rc, d = _fwd_plan("cos_x", 0, [mk(0, vec1)], [mk(1, vec1)], [mk(2, vec1)])
    assert rc == 0 and d["path"] == 1 and d["shape"] == [8, 3 << 26]
    odd = ((1 << 31) + 1,)
    rc, d = _fwd_plan("cos_x", 0, [mk(0, odd)], [mk(1, odd)], [mk(2, odd)])
    assert rc == 0 and d["path"] == 2


def test_recompute_validation_on_the_host():
    L = B.lib()
    R, C = 64, 256
    base = 1 << 20
    count = [0]

    def full(shape=(R, C)):  # every view at an address range of its own
        count[0] += 1
        return _rowmajor(base + count[0] * (1 << 30), shape)

    op = P.bcast_op_lookup("tanh_xy_b")
    args = [full(), full(), full((R, 1))]
    grads = [full(), full(), full((R, 1))]

    def ws(op_id, a, adj, g, dt=0):
        return L.bcast_dual_backward_recompute_workspace(ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(a)),
                                                         B._views(a), ctypes.c_int32(len(adj)), B._views(adj),
                                                         ctypes.c_int32(len(g)), B._views(g), None)

    def run(op_id, a, adj, g, dt=0):
        return L.bcast_dual_backward_recompute(ctypes.c_int32(op_id), ctypes.c_int(dt), ctypes.c_int32(len(a)), B._views(a),
                                               ctypes.c_int32(len(adj)), B._views(adj), ctypes.c_int32(len(g)),
                                               B._views(g), None, ctypes.c_size_t(0), None, None)

    assert ws(op, args, [full()], grads) == 0  # row sums of 256 columns finish inside the main pass
    assert run(999, args, [full()], grads) == -1
    assert run(op, args[:2], [full()], grads) == -2
    assert run(op, args, [full(), full()], grads) == -2
    assert run(op, args, [full()], grads[:2]) == -2
    assert run(op, args, [full()], grads, dt=7) == -7
    assert run(op, args, [full((R, C + 1))], grads) == -6
    assert run(op, args, [full()], [full(), full(), full((1, C))]) == -6  # b is [R x 1]: its gradient too
    # the arity ops: planned like any other (the plan call launches nothing), but they have no
    # kernels for views with row strides of their own
    pt3 = P.bcast_op_lookup("prod_tanh_3")
    info = B.PlanInfo()

    def plan3(a):
        adj3, g3 = [full()], [full(), full(), full()]
        return L.bcast_dual_backward_recompute_plan(ctypes.c_int32(pt3), ctypes.c_int(0), ctypes.c_int32(3), B._views(a),
                                                    ctypes.c_int32(1), B._views(adj3), ctypes.c_int32(3), B._views(g3),
                                                    ctypes.byref(info), None)

    assert plan3([full(), full(), full()]) == 0 and info.path == 1 and info.specialized == 1
    padded = B.raw_view(base + (1 << 36), (R, C), (C + 8, 1))
    assert plan3([padded, full(), full()]) == -12
    # a transposed argument has no tiled layout: refused, the cached-plane path still serves it
    assert run(op, [B.raw_view(base, (R, C), (1, R)), full(), args[2]], [full()], grads) == -12


def test_absurd_extents_and_strides_are_refused():
    """Extents and strides that would wrap 64-bit index arithmetic never reach a kernel."""
    base = 1 << 20
    huge = B.raw_view(base, (1 << 31, 1 << 31), (0, 0))                # 2^62 virtual copies of one element
    far = B.raw_view(base + (1 << 34), (4, 4), (1 << 50, 1))            # rows 2^50 elements apart
    ok = lambda k: _rowmajor(base + (k + 2) * (1 << 34), (4, 4))
    assert _fwd_plan("cos_x", 0, [huge], [ok(1)], [ok(2)])[0] == -5
    assert _fwd_plan("cos_x", 0, [far], [ok(1)], [ok(2)])[0] == -10
    assert _fwd_plan("cos_x", 0, [ok(0)], [ok(1)], [ok(2)])[0] == 0


def test_recompute_plan_picks_the_fixed_pattern_kernels_at_the_benchmark_shapes():
    L = B.lib()
    slot = [0]

    def view(shape):
        slot[0] += 1
        return _rowmajor(slot[0] * (1 << 34), shape)

    def plan(op_name, shapes, out_shape, n_out, dt=0):
        op = P.bcast_op_lookup(op_name)
        args = [view(s) for s in shapes]
        nondiff = P.bcast_op_info(op)[2]
        grads = [view(s) for j, s in enumerate(shapes) if not (nondiff >> j) & 1]
        adj = [view(out_shape) for _ in range(n_out)]
        info = B.PlanInfo()
        rc = L.bcast_dual_backward_recompute_plan(ctypes.c_int32(op), ctypes.c_int(dt), ctypes.c_int32(len(args)), B._views(args),
                                                  ctypes.c_int32(n_out), B._views(adj), ctypes.c_int32(len(grads)),
                                                  B._views(grads), ctypes.byref(info), None)
        return rc, info.as_dict()

    H, Bt = 4096, 1024
    full, row, col = (H, Bt), (1, Bt), (H, 1)
    rc, d = plan("hmlstm_update", [full] * 6 + [full, row] + [col] * 4, full, 2)           # config 3
    assert rc == 0 and d["path"] == 1 and d["specialized"] == 1 and d["n_second_pass"] == 0 and d["rows_per_block"] == 1
    rc, d = plan("hmlstm_update", [full] * 6 + [row, row] + [col] * 4, full, 2, dt=1)     # configs 0 / 2 shapes, fp64
    assert rc == 0 and d["specialized"] == 1
    rc, d = plan("hmlstm_update", [full] * 6 + [row, row] + [col] * 3 + [full], full, 2)  # a full-shape "bias": another pattern
    assert rc == 0 and d["path"] == 1 and d["specialized"] == 0
    n = 8192
    rc, d = plan("branchy5", [(n, n), (n, n), (1, n), (n, 1), (1, 1)], (n, n), 1)         # config 4
    assert rc == 0 and d["specialized"] == 1 and d["n_second_pass"] == 3 and d["rows_per_block"] == 128
    rc, d = plan("tanh_xy_b", [(4096, 4096), (4096, 4096), (4096, 1)], (4096, 4096), 1)    # config 1
    assert rc == 0 and d["specialized"] == 1


def test_launching_wrappers_refuse_host_tensors():
    """A host pointer handed to a kernel would be a GPU memory fault, not an error code: the
    binding's launching calls check residency before anything reaches the library (the plan
    queries, which launch nothing, keep taking any addresses)."""
    x, y, b = _t(4, 6), _t(4, 6), _t(4, 1)
    out, parts = [_t(4, 6)], [_t(4, 6) for _ in range(3)]
    op = P.bcast_op_lookup("tanh_xy_b")
    assert P.bcast_dual_forward_plan(op, [x, y, b], out, parts)["path"] == 1
    with pytest.raises(ValueError):
        P.bcast_dual_forward(op, [x, y, b], out, parts)
    with pytest.raises(ValueError):
        P.bcast_dual_backward(out, parts, [_t(4, 6), _t(4, 6), _t(4, 1)])
    with pytest.raises(ValueError):
        P.bcast_dual_backward_recompute(op, [x, y, b], out, [_t(4, 6), _t(4, 6), _t(4, 1)])
    with pytest.raises(ValueError):
        P.PreparedForward(op, [x, y, b], out, parts)
    with pytest.raises(ValueError):
        P.broadcast("tanh_xy_b", x, y, b)


def test_rank3_problem_plans_as_slices_and_on_the_generic_kernels():
    """A problem that stays at rank 3 (an argument broadcast along the middle dim only) is a batch of
    two-dim slices for the tiled kernels: one block grid per slice, one main backward launch, reduced
    gradients kept or summed along the outer dim through the second pass.  Forced onto the generic
    kernels it takes vectors along the innermost dim where the views allow it, and reductions over long
    fibres are cut into chunks, which need workspace for their partial sums and one more small launch each."""
    T_, B_, H_ = 64, 256, 1024
    base = [1 << 40]

    def view(shape):
        base[0] += 1 << 32
        strides, acc = [], 1
        for n in reversed(shape):
            strides.append(acc if n > 1 else 0)
            acc *= n
        return B.raw_view(base[0], shape, tuple(reversed(strides)))

    full, rs, ss, ts = (T_, B_, H_), (T_, 1, H_), (1, B_, 1), (1, 1, 1)
    args = [view(full), view(full), view(rs), view(ss), view(ts)]
    outs, parts = [view(full)], [view(full) for _ in range(5)]
    adj, grads = [view(full)], [view(full), view(full), view(rs), view(ss), view(ts)]
    L = B.lib()
    info = B.PlanInfo()
    # tiled: 64 slices of [256 x 1024]; one row per block step, 256 blocks per slice
    rc, d = _fwd_plan("branchy5", 0, args, outs, parts)
    assert rc == 0 and d["path"] == 1 and d["ndim"] == 3 and d["shape"] == [T_, B_, H_] and d["vec"] == 4
    assert d["uniform_stride"] == 1 and d["grid_x"] == 1 and d["grid_y"] == T_ * B_
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                    ctypes.c_int32(5), B._views(grads), ctypes.byref(info), None)
    # the kernel compiled for branchy5's mix (2 full, 1 row-sum, 1 col-sum, 1 all-sum per slice) + the second pass
    assert rc == 0 and info.path == 1 and info.n_launches == 2 and info.specialized == 1 and info.n_second_pass == 3
    ws = L.bcast_dual_backward_workspace(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                         ctypes.c_int32(5), B._views(grads), None)
    assert 0 < ws < (1 << 24)
    rc = L.bcast_dual_backward(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts), ctypes.c_int32(5),
                               B._views(grads), None, ctypes.c_size_t(0), None, None)
    assert rc == -3  # the workspace is asked for before anything is launched
    # the recompute entry point takes the slices too
    op = P.bcast_op_lookup("branchy5")
    rc = L.bcast_dual_backward_recompute_plan(ctypes.c_int32(op), ctypes.c_int(0), ctypes.c_int32(5), B._views(args), ctypes.c_int32(1),
                                              B._views(adj), ctypes.c_int32(5), B._views(grads), ctypes.byref(info), None)
    assert rc == 0 and info.path == 1 and info.ndim == 3
    # a gradient shaped like one slice (summed over the outer dim only): generic kernels
    g2 = [view(full), view(full), view((1, B_, H_)), view(ss), view(ts)]
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                    ctypes.c_int32(5), B._views(g2), ctypes.byref(info), None)
    assert rc == 0 and info.path == 2
    # forced onto the generic kernels
    generic = P.Options(force_generic=1)
    rc, d = _fwd_plan("branchy5", 0, args, outs, parts, generic)
    assert rc == 0 and d["path"] == 2 and d["ndim"] == 3 and d["vec"] == 4
    rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                    ctypes.c_int32(5), B._views(grads), ctypes.byref(info), ctypes.byref(generic))
    # two elementwise launches, three reductions, each cut into chunks and followed by its final kernel
    assert rc == 0 and info.path == 2 and info.n_launches == 2 + 3 + 3
    ws = L.bcast_dual_backward_workspace(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                         ctypes.c_int32(5), B._views(grads), ctypes.byref(generic))
    assert 0 < ws < (1 << 22)  # 65536 x 2 partial sums of 8 bytes for the [T x 1 x H] gradient, a few KiB for the others
    # four dims that do not merge stay with the generic kernels
    f4, r4 = (6, 5, 4, 64), (6, 1, 4, 1)
    a4 = [view(f4), view(f4), view((1, 5, 1, 64)), view(r4), view((1, 1, 1, 1))]
    rc, d = _fwd_plan("branchy5", 0, a4, [view(f4)], [view(f4) for _ in range(5)])
    assert rc == 0 and d["path"] == 2 and d["ndim"] == 4


def test_backward_and_recompute_plans_for_rows_the_vector_does_not_fit():
    """Rows of an odd length keep the 16-byte vector (`ragged`) and the kernel compiled for the
    call's class mix, the one that finishes a row of 2 or 4 column chunks inside one block
    included; the recompute call keeps a fixed pattern for the op's own orientation only."""
    def views(R, C):
        k = [0]

        def mk(shape):
            k[0] += 1
            return _rowmajor(k[0] << 32, shape)
        return mk

    L = B.lib()
    info = B.PlanInfo()
    for C, ragged in ((4096, 0), (4095, 1)):
        mk = views(512, C)
        adj, parts = [mk((512, C))], [mk((512, C)) for _ in range(3)]
        grads = [mk((512, C)), mk((512, C)), mk((512, 1))]  # tanh(x*y + b): full, full, row sums
        rc = L.bcast_dual_backward_plan(ctypes.c_int(0), ctypes.c_int32(1), B._views(adj), B._views(parts),
                                        ctypes.c_int32(3), B._views(grads), ctypes.byref(info), None)
        d = info.as_dict()
        assert rc == 0 and d["path"] == 1 and d["vec"] == 4 and d["ragged"] == ragged and d["specialized"] == 1, d
        assert (d["grid_x"], d["n_launches"], d["n_second_pass"]) == (1, 1, 0), d
    op = P.bcast_op_lookup("tanh_xy_b")
    for shape_b, C, want in (((512, 1), 1024, (0, 1)), ((512, 1), 1023, (1, 1)), ((1, 1023), 1023, (1, 0))):
        mk = views(512, C)
        args = [mk((512, C)), mk((512, C)), mk(shape_b)]
        adj = [mk((512, C))]
        grads = [mk((512, C)), mk((512, C)), mk(shape_b)]
        rc = L.bcast_dual_backward_recompute_plan(ctypes.c_int32(op), ctypes.c_int(0), ctypes.c_int32(3), B._views(args),
                                                  ctypes.c_int32(1), B._views(adj), ctypes.c_int32(3), B._views(grads),
                                                  ctypes.byref(info), None)
        d = info.as_dict()
        assert rc == 0 and d["path"] == 1 and d["vec"] == 4 and (d["ragged"], d["specialized"]) == want, (shape_b, C, d)


def test_noalloc_backward_refuses_what_exceeds_its_scratch_array():
    """A call whose partial sums need more than the library's static scratch array holds is refused with
    BCAST_ERR_WORKSPACE_TOO_SMALL before anything is launched (the views point at addresses never touched)."""
    R, C = 1 << 15, 1 << 15
    view = lambda k: B.raw_view(4096 + k * (1 << 34), (R, C), (C, 1))
    grads = [B.raw_view(4096 + 9 * (1 << 34), (1, C), (C, 1))]
    opt = P.Options(bwd_row_steps=1)  # one row per block: a partial sum per row and column
    L = B.lib()
    need = L.bcast_dual_backward_workspace(ctypes.c_int(1), ctypes.c_int32(1), B._views([view(0)]), B._views([view(1)]),
                                           ctypes.c_int32(1), B._views(grads), ctypes.byref(opt))
    assert need > P.NOALLOC_SCRATCH_BYTES
    rc = L.bcast_dual_backward_noalloc(ctypes.c_int(1), ctypes.c_int32(1), B._views([view(0)]), B._views([view(1)]),
                                       ctypes.c_int32(1), B._views(grads), None, ctypes.byref(opt))
    assert rc == -8
    # validation comes first, as in bcast_dual_backward
    rc = L.bcast_dual_backward_noalloc(ctypes.c_int(7), ctypes.c_int32(1), B._views([view(0)]), B._views([view(1)]),
                                       ctypes.c_int32(1), B._views(grads), None, None)
    assert rc == -7
    header = open(os.path.join(ROOT, "include", "bcast_dual.h")).read()
    assert f"#define BCAST_NOALLOC_SCRATCH_BYTES ({P.NOALLOC_SCRATCH_BYTES >> 20}u << 20)" in header


def test_unfused_step_argument_checks():
    """bcast_unfused_step validates on the host before anything is launched (addresses never touched)."""
    L = B.lib()
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    op = P.bcast_op_lookup("tanh_xy_b")
    R, C = 64, 128
    assert L.bcast_unfused_workspace(i32(op), ctypes.c_int(0), ctypes.c_int64(R), ctypes.c_int64(C)) >= 8 * R * C * 4
    assert L.bcast_unfused_workspace(i32(P.bcast_op_lookup("cos_x")), ctypes.c_int(0), ctypes.c_int64(R), ctypes.c_int64(C)) == 0
    ptr = lambda n: (vp * n)(*[4096 * (k + 1) for k in range(n)])
    kinds = lambda *k: (i32 * len(k))(*k)
    n = i32()

    def call(op_id, dt, n_args, kind, n_out, n_grads, ws, ws_bytes):
        return L.bcast_unfused_step(i32(op_id), ctypes.c_int(dt), ctypes.c_int64(R), ctypes.c_int64(C), i32(n_args), ptr(max(n_args, 1)),
                                    kind, i32(n_out), ptr(1), ptr(1), i32(n_grads), ptr(max(n_grads, 1)), vp(ws), ctypes.c_size_t(ws_bytes),
                                    None, ctypes.byref(n))
    big = 1 << 40
    assert call(op, 0, 3, kinds(0, 0, 2), 1, 3, 0, big) == -3           # no workspace
    assert call(op, 0, 3, kinds(0, 0, 2), 1, 3, 4096, 1024) == -8        # workspace too small
    assert call(op, 0, 3, kinds(0, 0, 2), 1, 3, 4096 + 8, big) == -11    # workspace not 256-byte aligned
    assert call(op, 0, 2, kinds(0, 0), 1, 3, 4096, big) == -2            # argument count
    assert call(op, 0, 3, kinds(0, 0, 2), 1, 2, 4096, big) == -2         # gradient count
    assert call(op, 7, 3, kinds(0, 0, 2), 1, 3, 4096, big) == -7         # dtype
    assert call(op, 0, 3, kinds(0, 0, 5), 1, 3, 4096, big) == -5         # unknown argument kind
    assert call(P.bcast_op_lookup("cos_x"), 0, 1, kinds(0), 1, 1, 4096, big) == -12
    assert call(10 ** 6, 0, 3, kinds(0, 0, 2), 1, 3, 4096, big) == -1
    b5 = P.bcast_op_lookup("branchy5")
    assert call(b5, 0, 5, kinds(0, 1, 1, 2, 3), 1, 5, 4096, big) == -12  # B must be a full array
