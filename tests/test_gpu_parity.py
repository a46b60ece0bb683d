"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Branch ids bit-exact; fp32 within max(1e-5 |x|, 1e-6); fp64 within
max(1e-12 |x|, 1e-13)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1810_08297_amd as P
from paper_1810_08297_amd import inputs
from gpu_util import TOL, check_close, check_op, full_rank, gpu_backward, gpu_forward, to_dev

pytestmark = pytest.mark.gpu

DTYPES = [np.float32, np.float64]


def small_args(op, R, C, dtype, seed=0):
    rng = np.random.default_rng(1000 + seed)
    full, row, col, sc = (R, C), (1, C), (R, 1), (1, 1)
    shp = {
        "hmlstm_update": [full] * 6 + [row, row] + [col] * 4,
        "linear12": [full] * 6 + [row, row] + [col] * 4,
        "tanh_xy_b": [full, full, col],
        "branchy5": [full, full, row, col, sc],
        "update_c": [full] * 4 + [row, row],
        "cos_x": [full],
        "elementary4": [full],
        "scale_xt": [full, sc],
        "pair3": [full, sc, col],
    }[op]
    args = [rng.standard_normal(s).astype(dtype) for s in shp]
    if op in ("hmlstm_update", "linear12"):
        args[6] = (rng.random(shp[6]) < 0.4).astype(dtype)
        args[7] = (rng.random(shp[7]) < 0.5).astype(dtype)
    if op == "update_c":
        args[4] = (rng.random(shp[4]) < 0.4).astype(dtype)
        args[5] = (rng.random(shp[5]) < 0.5).astype(dtype)
    if op == "pair3":
        args[1] = (np.abs(args[1]) + 0.5).astype(dtype)
    if op == "elementary4":
        args[0] = (np.abs(args[0]) * 2 - 0.5).astype(dtype)  # log1p wants x > -1
    n_out = oracle.op_info(op)[1]
    adj = [rng.standard_normal(full).astype(dtype) for _ in range(n_out)]
    return args, adj


OPS = ["hmlstm_update", "tanh_xy_b", "branchy5", "update_c", "cos_x", "scale_xt", "pair3", "linear12", "elementary4"]
# several tiles, ragged tails, one row / one column / one element, rows wider than a block
SHAPES = [(1, 1), (1, 7), (5, 1), (3, 5), (64, 16), (7, 33), (129, 260), (2, 4100), (300, 1028), (1, 5000),
          (5, 2048), (3, 4096), (7, 3500)]  # rows of two to four (fp64: up to eight) column chunks


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
@pytest.mark.parametrize("op", OPS)
def test_ops_all_shapes(op, dtype):
    for k, (R, C) in enumerate(SHAPES):
        args, adj = small_args(op, R, C, dtype, seed=k)
        check_op(op, args, adj, what=f"[{R}x{C}] ", recompute="required")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_paper_broadcast_example_trailing_dims(dtype):
    """b.(A, alpha, a): a scalar and an n-vector against n x m (Sec. 2.1.1, Eq. 1);
    dims an argument lacks are trailing."""
    rng = np.random.default_rng(5)
    A = rng.standard_normal((6, 9)).astype(dtype)
    alpha = (np.abs(rng.standard_normal((1,))) + 0.5).astype(dtype)
    a = rng.standard_normal((6,)).astype(dtype)
    adj = [rng.standard_normal((6, 9)).astype(dtype) for _ in range(2)]
    check_op("pair3", [A, alpha, a], adj)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_strided_and_permuted_layouts(dtype):
    """Column-major, sliced and permuted views go through the same entry points."""
    R, C = 37, 52
    args, adj = small_args("branchy5", R, C, dtype, seed=77)

    def col_major(t, k):  # same values, transposed storage
        return t.t().contiguous().t() if t.dim() == 2 else t

    def sliced(t, k):     # every second element of a wider buffer
        if t.dim() != 2 or t.shape[1] == 1:
            return t
        wide = torch.empty(t.shape[0], t.shape[1] * 2 + 3, dtype=t.dtype, device=t.device)
        wide[:, 1:1 + 2 * t.shape[1]:2] = t
        return wide[:, 1:1 + 2 * t.shape[1]:2]

    def padded_rows(t, k):  # row stride larger than the row: still the tiled path
        if t.dim() != 2 or t.shape[1] == 1:
            return t
        wide = torch.empty(t.shape[0], t.shape[1] + 12, dtype=t.dtype, device=t.device)
        wide[:, :t.shape[1]] = t
        return wide[:, :t.shape[1]]

    for name, view in (("col-major", col_major), ("sliced", sliced), ("padded", padded_rows)):
        check_op("branchy5", args, adj, view=view, what=f"[{name}] ")
    args, adj = small_args("hmlstm_update", R, C, dtype, seed=78)
    check_op("hmlstm_update", args, adj, view=col_major, what="[col-major] ")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_rank3_and_rank4(dtype):
    rng = np.random.default_rng(9)
    # x (3,1,5,2) * t (1,4,1,2): nothing merges; gradients reduce over different dim sets
    x = rng.standard_normal((3, 1, 5, 2)).astype(dtype)
    t = rng.standard_normal((1, 4, 1, 2)).astype(dtype)
    adj = [rng.standard_normal((3, 4, 5, 2)).astype(dtype)]
    check_op("scale_xt", [x, t], adj)
    # rank 3 with a middle broadcast dim
    A = rng.standard_normal((6, 7, 8)).astype(dtype)
    B = rng.uniform(0.1, 2, (6, 7, 8)).astype(dtype)
    r = rng.standard_normal((1, 7, 1)).astype(dtype)
    s = rng.standard_normal((6, 1, 8)).astype(dtype)
    tt = rng.standard_normal((1, 1, 1)).astype(dtype)
    adj = [rng.standard_normal((6, 7, 8)).astype(dtype)]
    check_op("branchy5", [A, B, r, s, tt], adj)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_forced_generic_kernels_match(dtype):
    """The generic strided kernels on problems the tiled kernels normally take."""
    for op in ("hmlstm_update", "branchy5", "pair3"):
        args, adj = small_args(op, 45, 70, dtype, seed=3)
        check_op(op, args, adj, what="[generic] ", options=P.Options(force_generic=1))


@pytest.mark.parametrize("arity", [1, 2, 3, 5, 9, 18])
def test_prod_tanh_family(arity):
    xs, adj = inputs.prod_tanh_inputs(arity, 33, 100, seed=arity)
    xs = [x + np.float32(0.5) for x in xs]
    # the oracle's family name is "prod_tanh"; the library's is "prod_tanh_<N>"
    o_out, o_parts, o_br = oracle.forward("prod_tanh", xs)
    dev = [to_dev(x) for x in xs]
    fb = gpu_forward(f"prod_tanh_{arity}", dev)
    torch.cuda.synchronize()
    assert np.array_equal(fb.branch.cpu().numpy(), o_br)
    check_close(fb.outs[0].cpu().numpy(), o_out[0], "value")
    for k in range(arity):
        check_close(fb.partials[k].cpu().numpy(), o_parts[k], f"partial {k}")
    bb = gpu_backward([to_dev(adj[0])], fb.partials, [x.shape for x in xs])
    torch.cuda.synchronize()
    want = oracle.backward(adj, [p.cpu().numpy() for p in fb.partials], [x.shape for x in xs])
    for k in range(arity):
        check_close(bb.grads[k].cpu().numpy(), want[k], f"grad {k}")
    # recompute in reverse: no planes; also with one argument a row vector and one a scalar (the
    # pattern is then read at run time and two gradients are sums)
    adj_dev = [to_dev(adj[0])]
    rb = P.alloc_recompute(fb.op_id, dev, adj_dev, [x.shape for x in xs])
    assert P.bcast_dual_backward_recompute_plan(fb.op_id, dev, adj_dev, rb.grads)["specialized"] == 1
    P.bcast_dual_backward_recompute(fb.op_id, dev, adj_dev, rb.grads, rb.workspace)
    torch.cuda.synchronize()
    for k in range(arity):
        check_close(rb.grads[k].cpu().numpy(), want[k], f"recomputed grad {k}")
    if arity >= 3:  # at least one argument keeps the full shape
        xs2 = list(xs)
        xs2[0] = np.ascontiguousarray(xs[0][:1])       # [1 x 100]
        xs2[-1] = np.ascontiguousarray(xs[-1][:1, :1])  # [1 x 1]
        dev2 = [to_dev(x) for x in xs2]
        f2 = gpu_forward(f"prod_tanh_{arity}", dev2)
        shapes2 = [x.shape for x in xs2]
        b2 = gpu_backward(adj_dev, f2.partials, shapes2)
        torch.cuda.synchronize()
        want2 = oracle.backward(adj, [p.cpu().numpy() for p in f2.partials], shapes2)
        r2 = P.alloc_recompute(f2.op_id, dev2, adj_dev, shapes2)
        assert P.bcast_dual_backward_recompute_plan(f2.op_id, dev2, adj_dev, r2.grads)["specialized"] == 0
        P.bcast_dual_backward_recompute(f2.op_id, dev2, adj_dev, r2.grads, r2.workspace)
        torch.cuda.synchronize()
        for k in range(arity):
            check_close(b2.grads[k].cpu().numpy(), want2[k], f"broadcast arguments, grad {k}")
            check_close(r2.grads[k].cpu().numpy(), want2[k], f"broadcast arguments, recomputed grad {k}")


def test_absent_planes_and_skipped_gradients():
    """A NULL plane is not stored by forward and counts as zeros in backward; a NULL
    gradient is skipped."""
    args, adj = small_args("hmlstm_update", 40, 64, np.float32, seed=11)
    Nd = 10
    # c' does not depend on o, h, b_o: leave those planes out
    mask = [True] * 20
    for jd in (2, 5, 8):
        mask[0 * Nd + jd] = False
    dev = [to_dev(a) for a in args]
    sentinel = gpu_forward("hmlstm_update", dev)  # full set, for reference
    fb = gpu_forward("hmlstm_update", dev, partial_mask=mask)
    torch.cuda.synchronize()
    for k in range(20):
        if mask[k]:
            assert torch.equal(fb.partials[k], sentinel.partials[k])
    didx = oracle.diff_arg_indices("hmlstm_update", 12)
    shapes = [args[j].shape for j in didx]
    adj_dev = [to_dev(a) for a in adj]
    full = gpu_backward(adj_dev, sentinel.partials, shapes)
    lean = gpu_backward(adj_dev, fb.partials, shapes)
    torch.cuda.synchronize()
    for a, b in zip(full.grads, lean.grads):
        assert torch.equal(a, b)
    want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in fb.partials], shapes)
    for k in range(Nd):
        check_close(lean.grads[k].cpu().numpy(), want[k], f"grad {k}")
    # skipped gradients stay untouched
    bb = P.alloc_backward(adj_dev, fb.partials, shapes)
    for g in bb.grads:
        g.fill_(123.0)
    keep = list(bb.grads)
    bb.grads = [g if k % 2 == 0 else None for k, g in enumerate(bb.grads)]
    bb.run(adj_dev, fb.partials)
    torch.cuda.synchronize()
    for k in range(Nd):
        if k % 2 == 0:
            assert torch.equal(keep[k], lean.grads[k])
        else:
            assert bool((keep[k] == 123.0).all())


def test_values_only_forward():
    args, _ = small_args("branchy5", 20, 24, np.float32, seed=2)
    dev = [to_dev(a) for a in args]
    ref = gpu_forward("branchy5", dev)
    fb = P.alloc_forward("branchy5", dev, want_branch=False, want_partials=False)
    fb.run(dev)
    torch.cuda.synchronize()
    assert torch.equal(fb.outs[0], ref.outs[0])


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_second_pass_geometries(dtype):
    """Row sums across several column tiles, column sums across several row tiles and the
    full sum across all blocks, with non-zero data for the scalar gradient."""
    rng = np.random.default_rng(21)
    R, C = 200, 2304  # > 1 column tile in both dtypes, > 1 row tile once rows sum
    x = rng.standard_normal((R, C)).astype(dtype)
    t = rng.standard_normal((1, 1)).astype(dtype)
    adj = [rng.standard_normal((R, C)).astype(dtype)]
    fb, bb = check_op("scale_xt", [x, t], adj)
    info = P.bcast_dual_backward_plan([to_dev(adj[0])], fb.partials, bb.grads)
    assert info["n_second_pass"] == 1 and info["grid_x"] > 1  # x, adj, plane merge to one long row
    args, adj = small_args("branchy5", R, C, dtype, seed=4)
    fb, bb = check_op("branchy5", args, adj)
    info = P.bcast_dual_backward_plan([to_dev(adj[0])], fb.partials, bb.grads)
    assert info["n_second_pass"] == 3 and info["grid_x"] > 1 and info["grid_y"] > 1
    # cancellation-heavy sums: large terms that cancel to O(1)
    big = (rng.standard_normal((R, C)) * 1e4).astype(dtype)
    Pl = rng.standard_normal((R, C)).astype(dtype)
    big[:, C // 2:] = -big[:, :C // 2]
    Pl[:, C // 2:] = Pl[:, :C // 2] * (1 + rng.standard_normal((R, C // 2)) * 1e-3).astype(dtype)
    g = gpu_backward([to_dev(big)], [to_dev(Pl)] * 3, [(R, 1), (1, C), (1, 1)])
    torch.cuda.synchronize()
    want = oracle.backward([big], [Pl] * 3, [(R, 1), (1, C), (1, 1)], threads=8)
    for k in range(3):
        check_close(g.grads[k].cpu().numpy(), want[k], f"cancelling sum {k}")
    if dtype == np.float64:
        # 2^70 + 40 ones - 2^70: exact only if partial sums carry more than a double's 53 bits
        n = 40
        a = np.ones((1, n + 2)); q = np.ones((1, n + 2))
        a[0, 0], q[0, 0], a[0, -1], q[0, -1] = 2.0 ** 35, 2.0 ** 35, -(2.0 ** 35), 2.0 ** 35
        for aa, qq in ((a, q), (a.T.copy(), q.T.copy())):
            g = gpu_backward([to_dev(aa)], [to_dev(qq)], [(1, 1)])
            torch.cuda.synchronize()
            assert float(g.grads[0].cpu()[0, 0]) == float(n)


def test_tuned_launch_shapes_agree():
    """Any rows-per-block choice, either assignment of rows to blocks and either tile order
    give results within tolerance of the oracle."""
    args, adj = small_args("branchy5", 333, 1100, np.float32, seed=6)
    for bwd_steps in (1, 7, 256):
        for interleave, reverse in ((1, 1), (0, 0), (1, 2), (0, 2)):
            check_op("branchy5", args, adj, what=f"[row steps {bwd_steps} interleave {interleave} reverse {reverse}] ",
                     options=P.Options(bwd_row_steps=bwd_steps, interleave_rows=interleave, reverse_tiles=reverse))
    first_to_last = P.Options(interleave_rows=0, reverse_tiles=0)
    for op, R, C in (("hmlstm_update", 300, 1028), ("tanh_xy_b", 129, 260)):
        a2, j2 = small_args(op, R, C, np.float64, seed=8)
        check_op(op, a2, j2, what="[contiguous rows, first to last] ", options=first_to_last)
    check_op("branchy5", args, adj, what="[plain stores] ", options=first_to_last.replace(nontemporal_stores=0))


def test_run_to_run_bitwise_determinism():
    op, args, adj = inputs.config_inputs(4, scale=1 / 8)
    dev = [to_dev(a) for a in args]
    adj_dev = [to_dev(a) for a in adj]
    runs = []
    for _ in range(2):
        fb = gpu_forward(op, dev)
        bb = gpu_backward(adj_dev, fb.partials, [a.shape for a in args])
        torch.cuda.synchronize()
        runs.append([t.clone() for t in fb.outs + fb.partials + bb.grads])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


# ---- the five benchmark configurations ---------------------------------------------------
@pytest.mark.parametrize("index", [0, 2])
def test_config_small_full(index):
    op, args, adj = inputs.config_inputs(index)
    fb, _ = check_op(op, args, adj, threads=16)
    br = fb.branch.cpu().numpy()
    hist = np.bincount(br.ravel(), minlength=3) / br.size
    assert hist[2] > 0.2 and hist[1] > 0.05 and hist[0] > 0.05  # all three branches occur


def test_config1_full_size():
    op, args, adj = inputs.config_inputs(1)
    check_op(op, args, adj, threads=16)


@pytest.mark.parametrize("p_index", [0, 1, 2])
def test_config3_full_size(p_index):
    op, args, adj = inputs.config_inputs(3, p_index=p_index)
    fb, _ = check_op(op, args, adj, threads=16)
    br = fb.branch.cpu().numpy()
    p = inputs.P_SWEEP[p_index]
    assert abs((br == 2).mean() - p) < 0.01


def _config4_every_element(dtype):
    """Config 4 at its full 8192 x 8192, in the launch geometry the benchmark times: every value, every
    element of the five planes, every branch id and every gradient (g_A, g_B full shape, g_r column sums,
    g_s row sums, g_t) against the oracle."""
    op, args, adj = inputs.config_inputs(4, dtype=dtype)
    fb, bb = check_op(op, args, adj, threads=16, recompute="required")
    # d out / d t is identically zero: the scalar gradient is exactly 0
    assert float(bb.grads[4].item()) == 0.0
    assert bool((fb.partials[4] == 0).all())
    br = fb.branch.cpu().numpy()
    assert 0.01 < br.mean() < 0.99  # both branches occur (how often depends on the drawn threshold t)


def test_config4_full_size_fp32():
    _config4_every_element(np.float32)


def test_config4_full_size_fp64():
    _config4_every_element(np.float64)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_config4_quarter_size_every_element(dtype):
    op, args, adj = inputs.config_inputs(4, dtype=dtype, scale=1 / 4)
    check_op(op, args, adj, threads=16)


def test_full_sum_at_bench_scale():
    """Scalar gradient with non-zero data over 16.8 M elements, every block's partial in play."""
    rng = np.random.default_rng(8)
    x = rng.standard_normal((4096, 4096)).astype(np.float32)
    t = rng.standard_normal((1, 1)).astype(np.float32)
    adj = [rng.standard_normal((4096, 4096)).astype(np.float32)]
    check_op("scale_xt", [x, t], adj, threads=16)


def test_end_to_end_against_wide_oracle_reports_cancellation():
    """Oracle forward -> backward entirely in wide precision vs GPU forward -> backward.
    Full-shape gradients meet the tolerance; a reduced gradient inherits the fp32 rounding
    of every stored plane, so it is held to tolerance relative to sum |terms| instead."""
    op, args, adj = inputs.config_inputs(3, scale=1 / 4)
    o_out, o_parts, _ = oracle.forward(op, args, threads=16)
    didx = oracle.diff_arg_indices(op, 12)
    want = oracle.backward(adj, o_parts, [args[j].shape for j in didx], threads=16)
    dev = [to_dev(a) for a in args]
    fb = gpu_forward(op, dev)
    bb = gpu_backward([to_dev(a) for a in adj], fb.partials, [args[j].shape for j in didx])
    torch.cuda.synchronize()
    # A full-shape gradient is sum_i adj_i * P_ij over the M = 2 outputs.  Each stored plane may differ
    # from the oracle's by its own tolerance max(1e-5 |P|, 1e-6), so the gradient may differ by
    # sum_i |adj_i| x that, plus the rounding of the fp32 result: the tolerance of a derived quantity,
    # not a relaxation of the planes' (which the parity tests hold to 1e-5 / 1e-6 themselves).
    rtol, atol = 1e-5, 1e-6
    for k in range(6):
        tol = sum(np.abs(adj[i].astype(np.float64)) * np.maximum(rtol * np.abs(o_parts[i * 10 + k].astype(np.float64)), atol)
                  for i in range(2)) + 1e-7 * np.abs(want[k].astype(np.float64))
        err = np.abs(bb.grads[k].cpu().numpy().astype(np.float64) - want[k].astype(np.float64))
        assert np.all(err <= tol), f"end-to-end grad {k}: worst err/tol {np.max(err / tol):.3f}"
    absP = [np.abs(p) for p in o_parts]
    absA = [np.abs(a) for a in adj]
    for k in range(6, 10):
        scale = oracle.backward(absA, absP, [args[j].shape for j in didx], threads=16)[k]
        err = np.abs(bb.grads[k].cpu().numpy().astype(np.float64) - want[k])
        assert np.all(err <= 1e-6 * scale + 1e-6)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_lean_plane_layout_gives_identical_results(dtype):
    """Identical planes stored once and always-zero planes left out: same outputs, same
    gradients, bit for bit, and the gradients still match the oracle."""
    op, args, adj = inputs.config_inputs(2, dtype=dtype)
    dev = [to_dev(a) for a in args]
    adj_dev = [to_dev(a) for a in adj]
    didx = oracle.diff_arg_indices(op, 12)
    shapes = [args[j].shape for j in didx]
    full = P.alloc_forward(op, dev).run(dev)
    lean = P.alloc_forward(op, dev, lean=True).run(dev)
    alias = P.bcast_op_plane_alias(lean.op_id)
    assert sum(p is None for p in lean.partials) == 3
    assert len({p.data_ptr() for p in lean.partials if p is not None}) == 10
    gf = P.alloc_backward(adj_dev, full.partials, shapes).run(adj_dev, full.partials)
    gl = P.alloc_backward(adj_dev, lean.partials, shapes).run(adj_dev, lean.partials)
    info = P.bcast_dual_backward_plan(adj_dev, lean.partials, gl.grads)
    assert info["path"] == 1 and info["specialized"] == 1  # shared planes loaded once, zero planes skipped
    assert P.bcast_dual_backward_plan(adj_dev, full.partials, gf.grads)["specialized"] == 1
    torch.cuda.synchronize()
    for a, b in zip(full.outs, lean.outs):
        assert torch.equal(a, b)
    for k, a in enumerate(alias):
        if a >= 0:
            assert torch.equal(full.partials[k], lean.partials[k])
        else:
            assert bool((full.partials[k] == 0).all())
    for a, b in zip(gf.grads, gl.grads):
        assert torch.equal(a, b)
    want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in lean.partials], shapes, threads=16)
    for k in range(10):
        check_close(gl.grads[k].cpu().numpy(), want[k], f"lean grad {k}")
    # branchy5: the plane of the threshold t is always zero
    op, args, adj = inputs.config_inputs(4, dtype=dtype, scale=1 / 16)
    dev = [to_dev(a) for a in args]
    lean = P.alloc_forward(op, dev, lean=True).run(dev)
    assert lean.partials[4] is None
    gl = P.alloc_backward([to_dev(adj[0])], lean.partials, [a.shape for a in args]).run([to_dev(adj[0])], lean.partials)
    torch.cuda.synchronize()
    want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in lean.partials],
                           [a.shape for a in args], threads=16)
    for k in range(5):
        check_close(gl.grads[k].cpu().numpy(), want[k], f"branchy5 lean grad {k}")


def test_recompute_refuses_what_it_cannot_do_and_skips_null_gradients():
    # four dims of which no two merge: only the plane-reading path has generic kernels
    rng = np.random.default_rng(4)
    x = to_dev(rng.standard_normal((3, 1, 5, 1)).astype(np.float32))
    t = to_dev(rng.standard_normal((1, 4, 1, 6)).astype(np.float32))
    adj = to_dev(rng.standard_normal((3, 4, 5, 6)).astype(np.float32))
    op = P.bcast_op_lookup("scale_xt")
    with pytest.raises(P.BcastError) as e:
        P.bcast_dual_backward_recompute(op, [x, t], [adj], [torch.empty_like(x), torch.empty_like(t)])
    assert e.value.status == -12
    with pytest.raises(P.BcastError) as e:  # the arity ops have no kernels for views with row strides of their own
        wide = to_dev(rng.standard_normal((4, 16)).astype(np.float32))
        xs = [wide[:, :8]] + [to_dev(rng.standard_normal((4, 8)).astype(np.float32)) for _ in range(2)]
        P.bcast_dual_backward_recompute(P.bcast_op_lookup("prod_tanh_3"), xs, [xs[1]], [torch.empty_like(xs[1]) for _ in xs])
    assert e.value.status == -12
    # a NULL gradient is skipped, the others are unaffected
    args, adjn = small_args("branchy5", 33, 260, np.float32, seed=9)
    dev = [to_dev(a) for a in args]
    adj_dev = [to_dev(adjn[0])]
    op = P.bcast_op_lookup("branchy5")
    full = P.alloc_recompute(op, dev, adj_dev, [a.shape for a in args])
    P.bcast_dual_backward_recompute(op, dev, adj_dev, full.grads, full.workspace)
    part = P.alloc_recompute(op, dev, adj_dev, [a.shape for a in args])
    sentinel = part.grads[1]
    sentinel.fill_(7.0)
    grads = list(part.grads)
    grads[1] = None
    P.bcast_dual_backward_recompute(op, dev, adj_dev, grads, part.workspace)
    torch.cuda.synchronize()
    assert bool((sentinel == 7.0).all())
    for k in (0, 2, 3, 4):
        assert torch.equal(grads[k], full.grads[k])


def test_recompute_fixed_and_runtime_patterns_agree():
    """The recompute kernel compiled for the op's usual broadcast pattern and the one that
    reads the gradient classes at run time give the same bits."""
    for op, idx in (("hmlstm_update", 2), ("branchy5", 4)):
        _, args, adj = inputs.config_inputs(idx, scale=1 / 4 if idx == 4 else 1.0)
        dev = [to_dev(a) for a in args]
        adj_dev = [to_dev(a) for a in adj]
        op_id = P.bcast_op_lookup(op)
        shapes = [args[j].shape for j in P.diff_arg_indices(op_id)]
        a = P.alloc_recompute(op_id, dev, adj_dev, shapes)
        P.bcast_dual_backward_recompute(op_id, dev, adj_dev, a.grads, a.workspace)
        table = P.Options(runtime_table=1)
        b = P.alloc_recompute(op_id, dev, adj_dev, shapes, options=table)
        P.bcast_dual_backward_recompute(op_id, dev, adj_dev, b.grads, b.workspace, options=table)
        torch.cuda.synchronize()
        for x, y in zip(a.grads, b.grads):
            if x.numel() == args[0].size or op == "hmlstm_update":
                assert torch.equal(x, y)
            else:  # sums taken with a different number of rows per block may round differently
                check_close(x.cpu().numpy(), y.cpu().numpy(), f"{op} reduced gradient")


def test_recompute_with_expanded_and_control_input_forms():
    """The fixed-pattern recompute kernels take an argument's broadcast form from its
    gradient's class; an argument that is a stride-0 expansion of a smaller array has a
    full-shape gradient but not a full-shape layout and must still be read correctly.  Control
    inputs (no gradient) are read in whatever form they come: row vector, column vector,
    scalar, full shape."""
    rng = np.random.default_rng(31)
    R, C = 96, 516
    x_row = rng.standard_normal((1, C)).astype(np.float32)
    y = rng.standard_normal((R, C)).astype(np.float32)
    b = rng.standard_normal((R, 1)).astype(np.float32)
    adj = [rng.standard_normal((R, C)).astype(np.float32)]
    x_full = np.ascontiguousarray(np.broadcast_to(x_row, (R, C)))
    o_out, o_parts, _ = oracle.forward("tanh_xy_b", [x_full, y, b], threads=8)
    want = oracle.backward(adj, o_parts, [(R, C), (R, C), (R, 1)], threads=8)
    dev = [to_dev(x_row).expand(R, C), to_dev(y), to_dev(b)]
    adj_dev = [to_dev(adj[0])]
    op_id = P.bcast_op_lookup("tanh_xy_b")
    rb = P.alloc_recompute(op_id, dev, adj_dev, [(R, C), (R, C), (R, 1)])
    P.bcast_dual_backward_recompute(op_id, dev, adj_dev, rb.grads, rb.workspace)
    torch.cuda.synchronize()
    for k, (g, w) in enumerate(zip(rb.grads, want)):
        check_close(g.cpu().numpy().reshape(w.shape), w, f"expanded x: recomputed gradient {k}")
    # HM-LSTM update with the two control inputs in every form
    op_id = P.bcast_op_lookup("hmlstm_update")
    forms = {"row": (1, C), "col": (R, 1), "scalar": (1, 1), "full": (R, C)}
    for zf, zbf in (("row", "row"), ("full", "row"), ("col", "scalar"), ("scalar", "col"), ("row", "full")):
        args, adj2 = small_args("hmlstm_update", R, C, np.float32, seed=40)
        args[6] = (rng.random(forms[zf]) < 0.4).astype(np.float32)
        args[7] = (rng.random(forms[zbf]) < 0.5).astype(np.float32)
        check_op("hmlstm_update", args, adj2, what=f"[z {zf}, z_below {zbf}] ", recompute="required")


@pytest.mark.parametrize("op,R,C", [("hmlstm_update", 64, 16), ("branchy5", 300, 1100), ("tanh_xy_b", 257, 515)])
def test_graph_replays_match_eager(op, R, C):
    """Forward + backward (+ the fixed-order second pass where one runs) captured into one HIP
    graph: the library allocates nothing, clears nothing with memset nodes and never
    synchronises, so every replay -- with new data in the same buffers and eager work in
    between -- must give the bits the eager calls give."""
    args0, adj0 = small_args(op, R, C, np.float32, seed=11)
    dev = [to_dev(a) for a in args0]
    adj_dev = [to_dev(a) for a in adj0]
    fb = P.alloc_forward(op, dev, want_branch=True)
    didx = oracle.diff_arg_indices(op, len(args0))
    gshapes = [args0[j].shape for j in didx]
    bb = P.alloc_backward(adj_dev, fb.partials, gshapes)
    fcall, bcall = fb.prepare(dev), bb.prepare(adj_dev, fb.partials)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fcall.launch()
        bcall.launch()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fcall.launch()
        bcall.launch()
    for rep in range(3):
        args_r, adj_r = small_args(op, R, C, np.float32, seed=20 + rep)
        for d, a in zip(dev, args_r):
            d.copy_(torch.from_numpy(a))
        for d, a in zip(adj_dev, adj_r):
            d.copy_(torch.from_numpy(a))
        # eager result first, kept aside; then poison the outputs and replay
        fcall.launch()
        bcall.launch()
        torch.cuda.synchronize()
        eager = [t.clone() for t in fb.outs + fb.partials + bb.grads] + [fb.branch.clone()]
        for t in fb.outs + fb.partials + bb.grads:
            t.fill_(float("nan"))
        fb.branch.fill_(255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        now = fb.outs + fb.partials + bb.grads + [fb.branch]
        for k, (e, n) in enumerate(zip(eager, now)):
            assert torch.equal(e, n), f"{op} replay {rep}: buffer {k} differs from the eager call"
        # and the replayed gradients are the oracle's
        want = oracle.backward(adj_r, [p.cpu().numpy() for p in fb.partials],
                               [full_rank(args_r[j], 2).shape for j in didx], threads=8)
        for k, (g, w) in enumerate(zip(bb.grads, want)):
            check_close(g.cpu().numpy().reshape(w.shape), w, f"{op} replay {rep} gradient {didx[k]}")


@pytest.mark.parametrize("op", ["hmlstm_update", "update_c", "tanh_xy_b", "branchy5"])
def test_unfused_baseline_computes_the_same_function(op):
    """The per-primitive comparison point timed by the benchmark is the same mathematical
    function: its outputs and reverse-mode gradients agree with the oracle's (looser line:
    library fp32 kernels, fp32 sums)."""
    from paper_1810_08297_amd.unfused_baseline import UnfusedStep
    args, adj = small_args(op, 130, 200, np.float32, seed=5)
    o_out, o_parts, _ = oracle.forward(op, args, threads=8)
    didx = oracle.diff_arg_indices(op, len(args))
    want = oracle.backward(adj, o_parts, [args[j].shape for j in didx], threads=8)
    outs, grads = UnfusedStep(op, [to_dev(a) for a in args], [to_dev(a) for a in adj]).run()
    for k, (g, w) in enumerate(zip(outs, o_out)):
        check_close(g.detach().cpu().numpy(), w, f"{op} unfused output {k}", rtol=1e-4, atol=1e-5)
    for k, (g, w) in enumerate(zip(grads, want)):
        scale = float(np.abs(w).max()) + 1.0
        check_close(g.cpu().numpy().reshape(w.shape), w, f"{op} unfused gradient {didx[k]}", rtol=1e-4, atol=1e-5 * scale)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
@pytest.mark.parametrize("op", ["hmlstm_update", "update_c", "tanh_xy_b", "branchy5"])
def test_unfused_primitive_kernels_match_the_oracle(op, dtype):
    """The library's per-primitive comparison system (one kernel per primitive, every branch computed and
    selected, reverse mode rule by rule) computes the oracle's function: values within the tolerance of
    every parity test; a full-shape gradient sum_i adj_i x dY_i/dX within sum_i |adj_i| x the tolerance of
    that partial (it is a different, longer chain of fp roundings than adjoint x stored plane, so the
    bound is the one of a derived quantity); a reduced gradient within tolerance x the sum of its terms'
    magnitudes.  Rows the 16-byte vector fits and rows it does not; control inputs per column and per element."""
    for R, C, per_element_z in ((300, 1100, False), (33, 1023, True)):
        args, adj = small_args(op, R, C, dtype, seed=R + C)
        if per_element_z and op in ("hmlstm_update", "update_c"):
            zi = 6 if op == "hmlstm_update" else 4
            args[zi] = (np.random.default_rng(R).random((R, C)) < 0.4).astype(dtype)
        _check_unfused(op, args, adj, dtype)


def _check_unfused(op, args, adj, dtype, threads=8):
    from paper_1810_08297_amd.unfused_baseline import UnfusedPrimitives
    rtol, atol = TOL[np.dtype(dtype)]
    R, C = adj[0].shape
    o_out, o_parts, _ = oracle.forward(op, args, threads=threads)
    didx = oracle.diff_arg_indices(op, len(args))
    nd, M = len(didx), len(o_out)
    shapes = [args[j].shape for j in didx]
    want = oracle.backward(adj, o_parts, shapes, threads=threads)
    absP = [np.abs(p.astype(np.float64)) for p in o_parts]
    absA = [np.abs(a.astype(np.float64)) for a in adj]
    sums = oracle.backward([a.astype(dtype) for a in absA], [p.astype(dtype) for p in absP], shapes, threads=threads)
    prog = UnfusedPrimitives(op, [to_dev(a) for a in args], [to_dev(a) for a in adj])
    outs, grads, n_kernels = prog.run()
    torch.cuda.synchronize()
    assert n_kernels >= {"hmlstm_update": 40, "update_c": 25, "tanh_xy_b": 6, "branchy5": 25}[op], n_kernels
    for k, (g, w) in enumerate(zip(outs, o_out)):
        check_close(g.cpu().numpy(), w, f"{op} [{R} x {C}] unfused output {k}")
    for k, (g, w) in enumerate(zip(grads, want)):
        got = g.cpu().numpy().astype(np.float64)
        err = np.abs(got - w.astype(np.float64))
        if shapes[k] == (R, C):
            tol = sum(absA[i] * np.maximum(rtol * absP[i * nd + k], atol) for i in range(M)) + 2 * np.finfo(dtype).eps * np.abs(w)
        else:
            tol = rtol * sums[k].astype(np.float64) + atol
        assert np.all(err <= tol), f"{op} [{R} x {C}] unfused gradient of argument {didx[k]}: worst err/tol {np.max(err / tol):.3f}"
    # run to run the same bits (fixed reduction orders, no atomics)
    first = [t.clone() for t in outs + grads]
    prog.run()
    torch.cuda.synchronize()
    for a, b in zip(first, outs + grads):
        assert torch.equal(a, b)


@pytest.mark.parametrize("index", [3, 1])
def test_unfused_primitive_kernels_at_benchmark_size(index):
    """The comparison system at the sizes `bench.py --unfused-baseline` times it (config 3: HM-LSTM update
    4096 x 1024 with per-element z; config 1: tanh(x*y + b) 4096 x 4096), every element against the oracle."""
    op, args, adj = inputs.config_inputs(index)
    _check_unfused(op, args, adj, np.float32, threads=16)


def _random_case(seed, dtype):
    """One random problem: an op with no control inputs, a random rank <= 4 output shape, every
    argument independently broadcast along a random subset of dims, and every device view
    randomly re-laid out (permuted storage order, padded rows, or every second element)."""
    rng = np.random.default_rng(9000 + seed)
    op = ["tanh_xy_b", "branchy5", "pair3", "scale_xt", "cos_x"][seed % 5]
    n_args = oracle.op_info(op)[0]
    nd = int(rng.integers(1, 5))
    shape = tuple(int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64])) for _ in range(nd))
    args = []
    for j in range(n_args):
        keep = rng.random(nd) < 0.6
        if j == 0:
            keep[:] = True  # one argument spans the whole output, so the unified shape is `shape`
        s = tuple(n if k else 1 for n, k in zip(shape, keep))
        a = rng.standard_normal(s).astype(dtype)
        if op == "pair3" and j == 1:
            a = (np.abs(a) + 0.5).astype(dtype)
        if op == "branchy5" and j == 1:
            a = rng.uniform(0.1, 2, s).astype(dtype)
        args.append(a)
    adj = [rng.standard_normal(shape).astype(dtype) for _ in range(oracle.op_info(op)[1])]
    styles = rng.integers(0, 4, n_args)

    def view(t, k):
        style = styles[k]
        if style == 1 and t.dim() >= 2:  # storage order reversed: the first dim is the contiguous one
            perm = list(range(t.dim()))[::-1]
            return t.permute(perm).contiguous().permute(perm)
        if style == 2 and t.dim() >= 1 and t.shape[-1] > 1:  # rows padded by three elements
            wide = torch.empty(*t.shape[:-1], t.shape[-1] + 3, dtype=t.dtype, device=t.device)
            wide[..., :t.shape[-1]] = t
            return wide[..., :t.shape[-1]]
        if style == 3 and t.dim() >= 1 and t.shape[-1] > 1:  # every second element of a wider buffer
            wide = torch.empty(*t.shape[:-1], 2 * t.shape[-1], dtype=t.dtype, device=t.device)
            wide[..., ::2] = t
            return wide[..., ::2]
        return t

    return op, args, adj, view, shape, styles


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_random_shapes_broadcast_patterns_and_layouts(dtype):
    for seed in range(60):
        op, args, adj, view, shape, styles = _random_case(seed, dtype)
        check_op(op, args, adj, view=view, what=f"[case {seed}: {op} {shape} layouts {list(styles)}] ")


def test_launch_events_time_one_kernel_only():
    """An event pair in the options is stamped by that call's main-pass launch only, and that
    launch computes what an ordinary launch computes."""
    op, args, adj = inputs.config_inputs(2)
    dev = [to_dev(a) for a in args]
    fb = P.alloc_forward(op, dev)
    fb.run(dev)
    torch.cuda.synchronize()
    plain = [t.clone() for t in fb.outs + fb.partials]
    for t in fb.outs + fb.partials:
        t.fill_(float("nan"))
    timer = P.LaunchTimer()
    P.bcast_dual_forward(fb.op_id, dev, fb.outs, fb.partials, fb.branch, options=timer.options())
    torch.cuda.synchronize()
    first = timer.ms()
    assert 1e-3 < first < 5.0, first  # config 2 forward: some 10 us
    for a, b in zip(plain, fb.outs + fb.partials):
        assert torch.equal(a, b)
    fb.run(dev)  # a call without the pair: the events keep the stamps of the first launch
    torch.cuda.synchronize()
    assert timer.ms() == first
    # backward: the main kernel takes the pair, the second reduction pass does not
    a4, j4 = small_args("branchy5", 300, 1100, np.float32, seed=2)
    d4, dj = [to_dev(a) for a in a4], [to_dev(a) for a in j4]
    f4 = P.alloc_forward("branchy5", d4).run(d4)
    bb = P.alloc_backward(dj, f4.partials, [a.shape for a in a4])
    bb.run(dj, f4.partials)
    torch.cuda.synchronize()
    ref = [g.clone() for g in bb.grads]
    P.bcast_dual_backward(dj, f4.partials, bb.grads, bb.workspace, options=timer.options())
    torch.cuda.synchronize()
    assert 1e-3 < timer.ms() < 5.0
    for a, b in zip(ref, bb.grads):
        assert torch.equal(a, b)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_predicate_ties_and_off_grid_control_values(dtype):
    """Branch decisions at their edges, bit-exact against the oracle: exact ties of strict
    comparisons (taken in the working precision), sums that round onto the threshold, control
    inputs that are neither 0 nor 1 (0.5, 2, -0.0, NaN fall to UPDATE unless z == 1)."""
    eps = np.finfo(dtype).eps
    # branchy5: A + s against t, around a tie and around a sum that rounds back onto A
    A = np.array([[0.5, 0.5, 0.5 + eps, 1.0, 1.0, 1.0 + 2 * eps, -3.0, 7.0]], dtype)
    s = np.array([[0.5]], dtype)
    t = np.array([[1.0]], dtype)
    B = np.full_like(A, 1.5)
    r = np.full_like(A, -0.75)
    check_op("branchy5", [A, B, r, s, t], [np.ones_like(A)], what="[tie] ")
    tiny = np.array([[eps / 4]], dtype)  # 1 + eps/4 rounds to 1: not greater than t = 1
    fb, _ = check_op("branchy5", [A, B, r, tiny, t], [np.ones_like(A)], what="[rounded sum] ")
    assert fb.branch.cpu().numpy().tolist()[0][3:6] == [0, 0, 1]
    # prod_tanh: x exactly 1/2 takes the else branch
    x = np.array([[0.5, np.nextafter(dtype(0.5), dtype(1)), np.nextafter(dtype(0.5), dtype(0)), 0.25, 0.75, -0.5]], dtype)
    xs = [x, x[:, ::-1].copy()]
    o_out, o_parts, o_br = oracle.forward("prod_tanh", xs)  # the library's name for arity 2 is prod_tanh_2
    fb = gpu_forward("prod_tanh_2", [to_dev(a) for a in xs])
    torch.cuda.synchronize()
    assert np.array_equal(fb.branch.cpu().numpy(), o_br) and o_br.tolist() == [[0, 2, 0, 0, 2, 0]]  # 1/2 itself counts as "not above"
    check_close(fb.outs[0].cpu().numpy(), o_out[0], "[g tie] value")
    for k in range(2):
        check_close(fb.partials[k].cpu().numpy(), o_parts[k], f"[g tie] partial {k}")
    # cell updates: every pair of control values from a set with off-grid members
    vals = np.array([0.0, 1.0, 0.5, 2.0, -0.0, np.nan, -1.0], dtype)
    z, zb = [m.reshape(1, -1).astype(dtype) for m in np.meshgrid(vals, vals, indexing="ij")]
    n = z.shape[1]
    rng = np.random.default_rng(12)
    full = lambda: rng.standard_normal((3, n)).astype(dtype)
    col = lambda: rng.standard_normal((3, 1)).astype(dtype)
    fb, _ = check_op("hmlstm_update", [full() for _ in range(6)] + [z, zb] + [col() for _ in range(4)], [full(), full()],
                     what="[control values] ")
    br = fb.branch.cpu().numpy()[0].reshape(len(vals), len(vals))
    assert (br[1] == 2).all()                     # z == 1: FLUSH whatever z_below is
    assert br[0, 0] == 1 and br[0, 4] == 1 and br[4, 0] == 1 and br[4, 4] == 1  # 0 and -0 are both zero: COPY
    assert br[0, 1] == 0 and br[2, 0] == 0 and br[5, 0] == 0 and br[0, 5] == 0 and br[3, 3] == 0  # the rest: UPDATE
    check_op("update_c", [full() for _ in range(4)] + [z, zb], [full()], what="[control values] ")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_saturating_and_tiny_inputs(dtype):
    """Gate pre-activations far into saturation (|x| up to 1e4), exact zeros, signed zeros and
    values near the underflow threshold: the stable forms of sigma, tanh and their derivatives
    must agree with the oracle's direct evaluation in long double."""
    tiny = np.finfo(dtype).tiny
    vals = np.array([-1e4, -100.0, -50.0, -20.0, -5.0, -1e-3, -tiny, -0.0, 0.0, tiny, 1e-3, 5.0, 20.0, 50.0, 100.0, 1e4], dtype)
    n = len(vals)
    rng = np.random.default_rng(77)
    pick = lambda: vals[rng.integers(0, n, (24, 4 * n))].astype(dtype)
    z = (rng.random((1, 4 * n)) < 0.4).astype(dtype)
    zb = (rng.random((1, 4 * n)) < 0.5).astype(dtype)
    small = lambda shape: (rng.standard_normal(shape) * 0.1).astype(dtype)
    adj = [rng.standard_normal((24, 4 * n)).astype(dtype) for _ in range(2)]
    c = rng.standard_normal((24, 4 * n)).astype(dtype)
    h = rng.standard_normal((24, 4 * n)).astype(dtype)
    check_op("hmlstm_update", [pick(), pick(), pick(), pick(), c, h, z, zb] + [small((24, 1)) for _ in range(4)], adj,
             what="[saturated gates] ")
    check_op("update_c", [c, pick(), pick(), pick(), z, zb], adj[:1], what="[saturated gates] ")
    # tanh(x*y + b): products from 1e-6 to 1e8
    x = pick()
    y = vals[rng.integers(0, n, (24, 1))].astype(dtype) * dtype(1e-2)
    check_op("tanh_xy_b", [x, np.broadcast_to(y, x.shape).copy(), small((24, 1))], adj[:1], what="[saturated tanh] ")
    # branchy5: exp(-A) from e^-80 to e^80, log1p(A^2) from A^2 = tiny to 1e8 (all finite in fp32)
    A = np.clip(pick(), -80, 80).astype(dtype)
    A[:, ::7] = vals[rng.integers(0, n, (24, A[:, ::7].shape[1]))]   # some |A| beyond the clip ...
    A[:, ::7] = np.abs(A[:, ::7])                                      # ... but only where exp(-A) underflows
    Bv = rng.uniform(0.1, 2, A.shape).astype(dtype)
    check_op("branchy5", [A, Bv, small((1, A.shape[1])), small((A.shape[0], 1)), np.zeros((1, 1), dtype)], adj[:1],
             what="[wide A] ")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_views_with_row_strides_of_their_own(dtype):
    """The usual framework layout: the four gate pre-activations are column slices of one
    [rows x 4 cols] buffer (row stride 4 cols) while c, h, the outputs and the planes are
    dense (row stride cols).  The tiled kernels address every view with its own row stride;
    gradients written into slices of a wider buffer likewise."""
    R, C = 130, 260
    rng = np.random.default_rng(91)
    gates = rng.standard_normal((R, 4 * C)).astype(dtype)
    f, i, o, g = [gates[:, k * C:(k + 1) * C] for k in range(4)]
    c, h = [rng.standard_normal((R, C)).astype(dtype) for _ in range(2)]
    z = (rng.random((R, 1)) < 0.4).astype(dtype)
    zb = (rng.random((R, 1)) < 0.5).astype(dtype)
    biases = [(rng.standard_normal((1, C)) * 0.1).astype(dtype) for _ in range(4)]
    args_np = [np.ascontiguousarray(a) for a in (f, i, o, g)] + [c, h, z, zb] + biases
    adj_np = [rng.standard_normal((R, C)).astype(dtype) for _ in range(2)]
    o_out, o_parts, o_br = oracle.forward("hmlstm_update", args_np, threads=8)

    gates_dev = to_dev(gates)
    dev = [gates_dev[:, k * C:(k + 1) * C] for k in range(4)] + [to_dev(a) for a in args_np[4:]]
    op_id = P.bcast_op_lookup("hmlstm_update")
    fb = P.alloc_forward("hmlstm_update", dev, want_branch=True)
    info = P.bcast_dual_forward_plan(op_id, dev, fb.outs, fb.partials)
    assert info["path"] == 1 and info["vec"] == (4 if dtype == np.float32 else 2)  # tiled, full vectors
    fb.run(dev)
    torch.cuda.synchronize()
    assert np.array_equal(fb.branch.cpu().numpy(), o_br)
    for k, (gv, w) in enumerate(zip(fb.outs, o_out)):
        check_close(gv.cpu().numpy(), w, f"output {k}")
    for k, (gv, w) in enumerate(zip(fb.partials, o_parts)):
        check_close(gv.cpu().numpy(), w, f"plane {k}")
    # backward: adjoints are slices of a wider buffer, gate gradients are written into slices of one
    adj_wide = to_dev(np.concatenate(adj_np + [np.zeros((R, 7), dtype)], axis=1))
    adj_dev = [adj_wide[:, :C], adj_wide[:, C:2 * C]]
    ggates = torch.full((R, 4 * C), float("nan"), dtype=gates_dev.dtype, device="cuda")
    grads = [ggates[:, k * C:(k + 1) * C] for k in range(4)] + [torch.empty((R, C), dtype=gates_dev.dtype, device="cuda")
                                                                for _ in range(2)] + \
            [torch.empty((1, C), dtype=gates_dev.dtype, device="cuda") for _ in range(4)]
    info = P.bcast_dual_backward_plan(adj_dev, fb.partials, grads)
    assert info["path"] == 1
    nbytes = P.bcast_dual_backward_workspace(adj_dev, fb.partials, grads)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    P.bcast_dual_backward(adj_dev, fb.partials, grads, ws)
    torch.cuda.synchronize()
    gshapes = [a.shape for a in args_np[:6]] + [b.shape for b in biases]
    want = oracle.backward(adj_np, [p.cpu().numpy() for p in fb.partials], gshapes, threads=8)
    for k, (gv, w) in enumerate(zip(grads, want)):
        check_close(gv.cpu().numpy(), w, f"gradient {k}")
    # the recompute entry point on the same views
    rgrads = [torch.empty_like(t) for t in grads]
    rg_wide = torch.empty((R, 4 * C), dtype=gates_dev.dtype, device="cuda")
    rgrads[:4] = [rg_wide[:, k * C:(k + 1) * C] for k in range(4)]
    nbytes = P.bcast_dual_backward_recompute_workspace(op_id, dev, adj_dev, rgrads)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    assert P.bcast_dual_backward_recompute_plan(op_id, dev, adj_dev, rgrads)["path"] == 1
    P.bcast_dual_backward_recompute(op_id, dev, adj_dev, rgrads, ws)
    torch.cuda.synchronize()
    for k, (gv, w) in enumerate(zip(rgrads, want)):
        check_close(gv.cpu().numpy(), w, f"recomputed gradient {k}")
    # an op without such kernels takes the generic ones and is still right
    xs = [to_dev(gates)[:, :C], to_dev(np.ascontiguousarray(c))]
    f2 = P.alloc_forward("prod_tanh_2", xs)
    assert P.bcast_dual_forward_plan(P.bcast_op_lookup("prod_tanh_2"), xs, f2.outs, f2.partials)["path"] == 2
    f2.run(xs)
    torch.cuda.synchronize()
    o2, p2, _ = oracle.forward("prod_tanh", [np.ascontiguousarray(f), c], threads=8)
    check_close(f2.outs[0].cpu().numpy(), o2[0], "prod_tanh_2 value")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_hmlstm_stored_batch_by_hidden(dtype):
    """The HM-LSTM update with every array transposed ([batch x hidden], biases [1 x hidden]): the
    bias gradients become sums over rows, taken by the kernels compiled for that mix (all planes
    stored, and the lean layout), with a second pass over many per-block partial sums."""
    op = "hmlstm_update"
    H, B = 520, 2100  # [2100 x 520]: a ragged last column chunk, row blocks that do not divide the rows
    args, adj = inputs.hmlstm_inputs(H, B, seed=77, dtype=dtype, z_per_element=True)
    args = [np.ascontiguousarray(a.T) for a in args]
    adj = [np.ascontiguousarray(a.T) for a in adj]
    bufs = check_op(op, args, adj, threads=16, what="batch x hidden")
    dev = [to_dev(a) for a in args]
    adj_dev = [to_dev(a) for a in adj]
    didx = oracle.diff_arg_indices(op, 12)
    shapes = [args[j].shape for j in didx]
    full = P.alloc_forward(op, dev).run(dev)
    lean = P.alloc_forward(op, dev, lean=True).run(dev)
    gf = P.alloc_backward(adj_dev, full.partials, shapes).run(adj_dev, full.partials)
    gl = P.alloc_backward(adj_dev, lean.partials, shapes).run(adj_dev, lean.partials)
    for parts, g in ((full.partials, gf), (lean.partials, gl)):
        info = P.bcast_dual_backward_plan(adj_dev, parts, g.grads)
        assert info["path"] == 1 and info["specialized"] == 1 and info["n_second_pass"] == 4
        assert info["rows_per_block"] > 1
    torch.cuda.synchronize()
    want = oracle.backward(adj, [p.cpu().numpy() for p in full.partials], shapes, threads=16)
    for k in range(10):
        check_close(gf.grads[k].cpu().numpy(), want[k], f"grad {k}")
        assert torch.equal(gf.grads[k], gl.grads[k])
    # recompute in reverse: the op's compiled-in broadcast pattern, transposed, is compiled in too
    rb = P.alloc_recompute(full.op_id, dev, adj_dev, shapes)
    assert P.bcast_dual_backward_recompute_plan(full.op_id, dev, adj_dev, rb.grads)["specialized"] == 1
    P.bcast_dual_backward_recompute(full.op_id, dev, adj_dev, rb.grads, rb.workspace)
    table = P.Options(runtime_table=1)
    r2 = P.alloc_recompute(full.op_id, dev, adj_dev, shapes, options=table)
    assert P.bcast_dual_backward_recompute_plan(full.op_id, dev, adj_dev, r2.grads, options=table)["specialized"] == 0
    P.bcast_dual_backward_recompute(full.op_id, dev, adj_dev, r2.grads, r2.workspace, options=table)
    torch.cuda.synchronize()
    for k in range(10):
        check_close(rb.grads[k].cpu().numpy(), want[k], f"recomputed grad {k}")
        assert torch.equal(rb.grads[k], r2.grads[k]), f"pattern fixed at compile time against run time, grad {k}"
    # many partial sums per output: one row per block leaves 2100 of them for the second pass
    g1 = P.alloc_backward(adj_dev, full.partials, shapes, options=P.Options(bwd_row_steps=1)).run(adj_dev, full.partials)
    torch.cuda.synchronize()
    for k in range(10):
        check_close(g1.grads[k].cpu().numpy(), want[k], f"one row per block, grad {k}")
    del bufs


def test_planes_beyond_4_gib():
    """33 300 x 32 768 fp32: every plane is 4.36 GB, so rows from 32 768 on lie beyond a 32-bit byte
    offset.  The tiled kernels take the problem (a lane's offset counts from its row step's first
    row); the oracle evaluates sampled rows on both sides of the 4 GiB line and sampled columns."""
    op, R, C = "branchy5", 33300, 32768
    if torch.cuda.mem_get_info()[0] < 100 * 2 ** 30:
        pytest.skip("needs 100 GiB of free device memory (an MI355X has 288 GB)")
    gen = torch.Generator(device="cuda").manual_seed(4321)
    A = torch.randn((R, C), device="cuda", generator=gen)
    Bm = torch.rand((R, C), device="cuda", generator=gen) * 1.9 + 0.1
    r = torch.randn((1, C), device="cuda", generator=gen)
    s = torch.randn((R, 1), device="cuda", generator=gen)
    t = torch.randn((1, 1), device="cuda", generator=gen)
    adj = torch.randn((R, C), device="cuda", generator=gen)
    dev = [A, Bm, r, s, t]
    shapes = [tuple(x.shape) for x in dev]
    fb = P.alloc_forward(op, dev, want_branch=True, staggered=False)
    assert P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, fb.branch)["path"] == 1
    fb.run(dev)
    bb = P.alloc_backward([adj], fb.partials, shapes, staggered=False)
    info = P.bcast_dual_backward_plan([adj], fb.partials, bb.grads)
    assert info["path"] == 1 and info["specialized"] == 1
    bb.run([adj], fb.partials)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 32767, 32768, 32769, R - 1], rng.integers(0, R, 8)]))
    cols = np.unique(np.concatenate([[0, C - 1], rng.integers(0, C, 6)]))
    ridx, cidx = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
    host = lambda x: x.cpu().numpy()
    sub = [host(A[ridx]), host(Bm[ridx]), host(r), host(s[ridx]), host(t)]
    o_out, o_parts, o_br = oracle.forward(op, sub, threads=16)
    assert np.array_equal(host(fb.branch[ridx]), o_br)
    check_close(host(fb.outs[0][ridx]), o_out[0], "value rows")
    planes_rows = [host(p[ridx]) for p in fb.partials]
    for k in range(5):
        check_close(planes_rows[k], o_parts[k], f"plane {k} rows")
    want = oracle.backward([host(adj[ridx])], planes_rows,
                           [(len(rows), C), (len(rows), C), (1, C), (len(rows), 1), (1, 1)], threads=16)
    planes_cols = [host(p[:, cidx]) for p in fb.partials]
    wantc = oracle.backward([host(adj[:, cidx])], planes_cols,
                            [(R, len(cols)), (R, len(cols)), (1, len(cols)), (R, 1), (1, 1)], threads=16)

    def check_grads(g, what):
        check_close(host(g[0][ridx]), want[0], f"{what} g_A rows")
        check_close(host(g[1][ridx]), want[1], f"{what} g_B rows")
        check_close(host(g[3][ridx]), want[3], f"{what} g_s rows")
        check_close(host(g[2][:, cidx]), wantc[2], f"{what} g_r cols")
        assert float(g[4].item()) == 0.0

    check_grads(bb.grads, "class kernel")
    # the kernel that reads the gradient table at run time
    table = P.Options(runtime_table=1)
    b2 = P.alloc_backward([adj], fb.partials, shapes, staggered=False, options=table)
    assert P.bcast_dual_backward_plan([adj], fb.partials, b2.grads, options=table)["specialized"] == 0
    b2.run([adj], fb.partials)
    torch.cuda.synchronize()
    check_grads(b2.grads, "run-time table")
    assert torch.equal(b2.grads[0], bb.grads[0]) and torch.equal(b2.grads[1], bb.grads[1])
    del b2
    # an adjoint with a row stride of its own (rows padded by 64 elements: 4.37 GB)
    wide = torch.empty((R, C + 64), device="cuda")
    adj_v = wide[:, :C]
    adj_v.copy_(adj)
    b3 = P.alloc_backward([adj_v], fb.partials, shapes, staggered=False)
    assert P.bcast_dual_backward_plan([adj_v], fb.partials, b3.grads)["path"] == 1
    b3.run([adj_v], fb.partials)
    torch.cuda.synchronize()
    check_grads(b3.grads, "padded adjoint")
    assert torch.equal(b3.grads[0], bb.grads[0]) and torch.equal(b3.grads[1], bb.grads[1])
    del b3, wide, adj_v
    # recompute in reverse: no planes at all
    for p_ in fb.partials:
        p_.zero_()
    rb = P.alloc_recompute(fb.op_id, dev, [adj], shapes, staggered=False)
    assert P.bcast_dual_backward_recompute_plan(fb.op_id, dev, [adj], rb.grads)["path"] == 1
    P.bcast_dual_backward_recompute(fb.op_id, dev, [adj], rb.grads, rb.workspace)
    torch.cuda.synchronize()
    check_grads(rb.grads, "recompute")


def test_long_vector_and_dims_too_long_to_fuse():
    """A dim of more than 2^28 elements is taken as rows of equal length (here 3 * 2^27 = 2 rows of
    201 326 592), and contiguous dims are fused only up to that length ([2048 x 1024 x 160] stays
    [2 097 152 x 160]): the scalar's gradient is a sum over all 402 653 184 / 335 544 320 elements."""
    op = "scale_xt"
    if torch.cuda.mem_get_info()[0] < 24 * 2 ** 30:
        pytest.skip("needs 24 GiB of free device memory")
    gen = torch.Generator(device="cuda").manual_seed(99)
    for shape, merged in (((3 << 27,), [2, 3 << 26]), ((2048, 1024, 160), [2048 * 1024, 160])):
        n = int(np.prod(shape))
        x = torch.randn(shape, device="cuda", generator=gen)
        t = torch.full((1,) * len(shape), 1.25, device="cuda")
        adj = torch.randn(shape, device="cuda", generator=gen)
        dev = [x, t]
        fb = P.alloc_forward(op, dev, staggered=False)
        info = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials)
        assert info["path"] == 1 and info["shape"] == merged, info
        fb.run(dev)
        bb = P.alloc_backward([adj], fb.partials, [tuple(x.shape), tuple(t.shape)], staggered=False)
        info = P.bcast_dual_backward_plan([adj], fb.partials, bb.grads)
        assert info["path"] == 1 and info["shape"] == merged, info
        bb.run([adj], fb.partials)
        torch.cuda.synchronize()
        flat = lambda z: z.reshape(-1)
        # elementwise results on slices at the start, across the middle (the seam of the two rows) and at the end
        for lo, hi in ((0, 4096), (n // 2 - 2048, n // 2 + 2048), (n - 4096, n)):
            sub = [flat(x)[lo:hi].cpu().numpy(), np.full((1,), 1.25, np.float32)]
            o_out, o_parts, _ = oracle.forward(op, sub, threads=4)
            check_close(flat(fb.outs[0])[lo:hi].cpu().numpy(), o_out[0], f"{shape} out [{lo}:{hi}]")
            for k in range(2):
                check_close(flat(fb.partials[k])[lo:hi].cpu().numpy(), o_parts[k], f"{shape} plane {k} [{lo}:{hi}]")
            want = oracle.backward([flat(adj)[lo:hi].cpu().numpy()], [flat(p_)[lo:hi].cpu().numpy() for p_ in fb.partials],
                                   [(hi - lo,), (hi - lo,)], threads=4)
            check_close(flat(bb.grads[0])[lo:hi].cpu().numpy(), want[0], f"{shape} g_x [{lo}:{hi}]")
        # the full sum, by the oracle over every element
        want = oracle.backward([flat(adj).cpu().numpy()], [flat(p_).cpu().numpy() for p_ in fb.partials], [(n,), (1,)], threads=16)
        check_close(bb.grads[1].cpu().numpy().reshape(1), want[1].reshape(1), f"{shape} g_t")
        # recompute in reverse takes the same split
        rb = P.alloc_recompute(fb.op_id, dev, [adj], [tuple(x.shape), tuple(t.shape)], staggered=False)
        P.bcast_dual_backward_recompute(fb.op_id, dev, [adj], rb.grads, rb.workspace)
        torch.cuda.synchronize()
        assert torch.equal(rb.grads[0], bb.grads[0])
        check_close(rb.grads[1].cpu().numpy().reshape(1), want[1].reshape(1), f"{shape} recomputed g_t")
        del x, adj, fb, bb, rb


def _random_2d_case(seed, dtype):
    """A 2-D problem of up to a few million elements -- several row tiles and column chunks, ragged
    edges -- with every argument's broadcast form (full, row vector, column vector, scalar) drawn at
    random, control inputs included, and some views with padded rows."""
    rng = np.random.default_rng(31000 + seed)
    op = ["hmlstm_update", "tanh_xy_b", "branchy5", "update_c", "pair3", "linear12"][seed % 6]
    n_args = oracle.op_info(op)[0]
    R = int(rng.choice([1, 7, 64, 255, 1000, 2047]))
    C = int(rng.choice([1, 5, 64, 260, 1024, 2048, 4100]))
    control = {"hmlstm_update": (6, 7), "linear12": (6, 7), "update_c": (4, 5)}.get(op, ())
    args = []
    for j in range(n_args):
        form = 0 if j == 0 else int(rng.choice([0, 0, 1, 2, 3]))  # the first argument spans the output
        s = [(R, C), (1, C), (R, 1), (1, 1)][form]
        if j in control:
            a = (rng.random(s) < 0.45).astype(dtype)
        else:
            a = rng.standard_normal(s).astype(dtype)
        if op == "pair3" and j == 1:
            a = (np.abs(a) + 0.5).astype(dtype)
        if op == "branchy5" and j == 1:
            a = rng.uniform(0.1, 2, s).astype(dtype)
        args.append(a)
    adj = [rng.standard_normal((R, C)).astype(dtype) for _ in range(oracle.op_info(op)[1])]
    padded = rng.random(n_args) < 0.25

    def view(t, k):
        if padded[k] and t.shape[-1] > 1:  # rows padded by eight elements: a row stride of its own
            wide = torch.empty(t.shape[0], t.shape[1] + 8, dtype=t.dtype, device=t.device)
            wide[:, :t.shape[1]] = t
            return wide[:, :t.shape[1]]
        return t

    return op, args, adj, view, (R, C), [a.shape for a in args]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_random_2d_problems_of_many_tiles(dtype):
    for seed in range(36):
        op, args, adj, view, shape, forms = _random_2d_case(seed, dtype)
        check_op(op, args, adj, view=view, threads=16, what=f"[case {seed}: {op} {shape} argument shapes {forms}] ")


def test_two_streams_run_independent_problems():
    """Calls enqueue only on the stream they are given and share no device state: two problems
    issued alternately on two streams (default priority) give, bit for bit, what each gives alone
    -- second reduction passes and their workspaces included."""
    cases = [("branchy5", 700, 2100, 3), ("hmlstm_update", 1500, 520, 4)]
    work = []
    for op, R, C, seed in cases:
        args, adj = small_args(op, R, C, np.float32, seed=seed)
        dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
        didx = oracle.diff_arg_indices(op, len(args))
        shapes = [args[j].shape for j in didx]
        fb = P.alloc_forward(op, dev)
        bb = P.alloc_backward(adj_dev, fb.partials, shapes)
        fb.run(dev)
        bb.run(adj_dev, fb.partials)
        torch.cuda.synchronize()
        alone = [t.clone() for t in fb.outs + fb.partials + bb.grads]
        work.append((dev, adj_dev, fb, bb, alone))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(5):
        for dev, adj_dev, fb, bb, _ in work:
            for t in fb.outs + fb.partials + bb.grads:
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        for k in range(2):  # forward calls first, then the backward calls, each on its problem's stream
            dev, adj_dev, fb, bb, _ = work[k]
            fb.run(dev, stream=streams[k])
        for k in (1, 0):
            dev, adj_dev, fb, bb, _ = work[k]
            bb.run(adj_dev, fb.partials, stream=streams[k])
        for s_ in streams:
            s_.synchronize()
        for dev, adj_dev, fb, bb, alone in work:
            for got, want in zip(fb.outs + fb.partials + bb.grads, alone):
                assert torch.equal(got, want), f"repetition {rep}"


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_planes_interleaved_by_row(dtype):
    """Outputs and planes interleaved by row in one slab (and the arguments, adjoints and gradients likewise,
    each group in a slab of its own): the groups have different row strides, the benchmark ops' mixes still get their
    compiled-per-mix backward kernel (built for views with strides of their own), and every result has the
    bits of the default layout."""
    for op, R, C, lean in (("hmlstm_update", 300, 1024, False), ("hmlstm_update", 130, 2052, True), ("branchy5", 260, 1100, False),
                           ("branchy5", 520, 2048, True), ("tanh_xy_b", 200, 4096, False), ("tanh_xy_b", 70, 1028, False)):
        args, adj = small_args(op, R, C, dtype, seed=R + C)
        dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
        shapes = [args[j].shape for j in oracle.diff_arg_indices(op, len(args))]
        ref = P.alloc_forward(op, dev, want_branch=True, lean=lean).run(dev)
        refb = P.alloc_backward(adj_dev, ref.partials, shapes).run(adj_dev, ref.partials)
        dev_i, _k1 = P.to_slab(dev, layout="interleaved")
        adj_i, _k2 = P.to_slab(adj_dev, layout="interleaved")
        fb = P.alloc_forward(op, dev_i, want_branch=True, lean=lean, layout="interleaved")
        assert fb.outs[0].stride(0) > C and not fb.outs[0].is_contiguous()
        fplan = P.bcast_dual_forward_plan(fb.op_id, dev_i, fb.outs, fb.partials, fb.branch)
        assert fplan["path"] == 1 and fplan["uniform_stride"] == 0
        fb.run(dev_i)
        bb = P.alloc_backward(adj_i, fb.partials, shapes, layout="interleaved")
        bplan = P.bcast_dual_backward_plan(adj_i, fb.partials, bb.grads)
        assert bplan["path"] == 1 and bplan["uniform_stride"] == 0
        if C % (16 // np.dtype(dtype).itemsize) == 0:  # the benchmark ops' mixes are also built for strides per view
            assert bplan["specialized"] == 1, (op, bplan)
        bb.run(adj_i, fb.partials)
        torch.cuda.synchronize()
        assert torch.equal(fb.branch, ref.branch)
        for k, (g, w) in enumerate(zip(fb.outs + [p for p in fb.partials if p is not None], ref.outs + [p for p in ref.partials if p is not None])):
            assert torch.equal(g, w), f"{op} output or plane {k}"
        for k, (g, w) in enumerate(zip(bb.grads, refb.grads)):
            if g.numel() == R * C:
                assert torch.equal(g, w), f"{op} gradient {k}"
            else:  # sums taken by another kernel may round differently
                check_close(g.cpu().numpy(), w.cpu().numpy(), f"{op} reduced gradient {k}")
        want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in fb.partials], shapes, threads=8)
        for k, (g, w) in enumerate(zip(bb.grads, want)):
            check_close(g.cpu().numpy(), w, f"{op} gradient {k} against the oracle")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_store_forms_give_identical_bits(dtype):
    """Plain stores, stores with the nontemporal hint, and a forward launch that changes from one to the other
    part way through its walk write the same bits: outputs, planes, branch ids and gradients of every class,
    on the kernels compiled per mix and on the one that reads the gradient table."""
    for op, R, C in (("hmlstm_update", 300, 1024), ("branchy5", 520, 2048), ("tanh_xy_b", 200, 1024), ("hmlstm_update", 70, 1028)):
        args, adj = small_args(op, R, C, dtype, seed=R + C)
        dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
        shapes = [args[j].shape for j in oracle.diff_arg_indices(op, len(args))]
        results = []
        for opt in (P.Options(nontemporal_stores=0), P.Options(nontemporal_stores=3, fwd_keep_mib=0, bwd_nt_min_mib=0),
                    P.Options(nontemporal_stores=3, fwd_keep_mib=1, bwd_nt_min_mib=0), P.Options(runtime_table=1, fwd_keep_mib=2)):
            fb = P.alloc_forward(op, dev, want_branch=True, options=opt)
            plan = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, fb.branch, options=opt)
            fb.run(dev)
            bb = P.alloc_backward(adj_dev, fb.partials, shapes, options=opt).run(adj_dev, fb.partials)
            torch.cuda.synchronize()
            results.append((plan["nontemporal_tiles"], fb.outs + fb.partials + [fb.branch] + bb.grads))
        tiles = [r[0] for r in results]
        assert tiles[0] == 0 and tiles[1] > tiles[2] > 0, tiles  # none, all, all but the last MiB
        for k in range(1, 3):
            for a, b in zip(results[0][1], results[k][1]):
                assert torch.equal(a, b), f"{op} [{R} x {C}] option set {k}"
        for a, b in zip(results[0][1][: -len(shapes)], results[3][1][: -len(shapes)]):
            assert torch.equal(a, b)
        for a, b in zip(results[0][1][-len(shapes):], results[3][1][-len(shapes):]):  # another kernel's sums may round differently
            check_close(a.cpu().numpy(), b.cpu().numpy(), f"{op} gradient, run-time table")


def test_two_host_threads_with_different_options():
    """The library holds no state between calls: two host threads, each launching its own problem on its own
    stream with options of its own (one forces the generic kernels and plain stores, the other the run-time
    table and 3 row steps per block), get bit for bit what each gets alone."""
    import threading
    cases = [("branchy5", 700, 2100, 3, P.Options(force_generic=1, nontemporal_stores=0)),
             ("hmlstm_update", 1500, 520, 4, P.Options(runtime_table=1, bwd_row_steps=3))]
    work = []
    for op, R, C, seed, opt in cases:
        args, adj = small_args(op, R, C, np.float32, seed=seed)
        dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
        shapes = [args[j].shape for j in oracle.diff_arg_indices(op, len(args))]
        fb = P.alloc_forward(op, dev, options=opt)
        bb = P.alloc_backward(adj_dev, fb.partials, shapes, options=opt)
        fb.run(dev)
        bb.run(adj_dev, fb.partials)
        torch.cuda.synchronize()
        alone = [t.clone() for t in fb.outs + fb.partials + bb.grads]
        want_path = 2 if opt.force_generic else 1
        assert P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, options=opt)["path"] == want_path
        work.append((dev, adj_dev, fb, bb, alone, torch.cuda.Stream()))
    for dev, adj_dev, fb, bb, _, _ in work:
        for t in fb.outs + fb.partials + bb.grads:
            t.fill_(float("nan"))
    torch.cuda.synchronize()
    errors = []

    def worker(k):
        try:
            dev, adj_dev, fb, bb, _, stream = work[k]
            for _ in range(20):
                fb.run(dev, stream=stream)
                bb.run(adj_dev, fb.partials, stream=stream)
            stream.synchronize()
        except Exception as e:  # noqa: BLE001 -- reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for dev, adj_dev, fb, bb, alone, _ in work:
        for got, want in zip(fb.outs + fb.partials + bb.grads, alone):
            assert torch.equal(got, want)


@pytest.mark.parametrize("planes", ["all", "lean", "none"])
def test_autograd_node_inside_a_reverse_mode_program(planes):
    """Mixed mode as Sec. 2.2.3 describes it: the fused broadcast is one node of a surrounding
    reverse-mode program (torch.autograd here).  The gradients that reach the program's leaves --
    through the node, a matmul before it and a weighted sum after it -- match those of the same
    program with the update written as per-primitive torch operations, and the node's own outputs
    and gradients match the oracle."""
    from paper_1810_08297_amd.unfused_baseline import FUNCTIONS
    torch.manual_seed(11)
    H, Bt, K = 96, 80, 24
    dev = "cuda"
    W = torch.randn(4 * H, K, device=dev, requires_grad=True)
    x = torch.randn(K, Bt, device=dev)
    c = torch.randn(H, Bt, device=dev, requires_grad=True)
    h = torch.randn(H, Bt, device=dev, requires_grad=True)
    z = (torch.rand(1, Bt, device=dev) < 0.4).float()
    zb = (torch.rand(Bt, device=dev) < 0.5).float()   # rank 1: aligned at the last dim, as torch does
    biases = [(0.1 * torch.randn(H, 1, device=dev)).requires_grad_() for _ in range(4)]
    wc, wh = torch.randn(H, Bt, device=dev), torch.randn(H, Bt, device=dev)

    def program(update):
        gates = W @ x                                    # [4H x B]: the gates are row slices of one buffer
        f, i, o, g = (gates[k * H:(k + 1) * H] for k in range(4))
        cn, hn = update(f, i, o, g, c, h, z, zb, *biases)
        return cn, hn, (cn * wc).sum() + (hn * wh).sum()

    leaves = [W, c, h] + biases
    cn1, hn1, loss1 = program(lambda *a: P.broadcast("hmlstm_update", *a, planes=planes))
    g1 = torch.autograd.grad(loss1, leaves)
    cn2, hn2, loss2 = program(FUNCTIONS["hmlstm_update"][0])
    g2 = torch.autograd.grad(loss2, leaves)
    torch.cuda.synchronize()
    for a, b, what in ((cn1, cn2, "c'"), (hn1, hn2, "h'")):
        assert torch.allclose(a, b, rtol=1e-5, atol=1e-6), what
    for a, b, leaf in zip(g1, g2, ["W", "c", "h", "b_f", "b_i", "b_o", "b_g"]):
        assert a.shape == b.shape
        assert torch.allclose(a, b, rtol=2e-4, atol=2e-5), (leaf, float((a - b).abs().max()))  # a K = 24 matmul follows
    # the node alone against the oracle: values, and the gradients for the adjoints wc, wh
    gates = (W @ x).detach()
    args = [gates[k * H:(k + 1) * H].contiguous() for k in range(4)] + [c.detach(), h.detach(), z, zb.reshape(1, Bt)] + \
           [b_.detach() for b_ in biases]
    host = [a.cpu().numpy() for a in args]
    o_out, o_parts, _ = oracle.forward("hmlstm_update", host, threads=8)
    check_close(cn1.detach().cpu().numpy(), o_out[0], "node c'")
    check_close(hn1.detach().cpu().numpy(), o_out[1], "node h'")
    leaf_args = [a.clone().requires_grad_(k not in (6, 7)) for k, a in enumerate(args)]
    outs = P.broadcast("hmlstm_update", *leaf_args, planes=planes)
    got = torch.autograd.grad(outs, [a for a in leaf_args if a.requires_grad], [wc, wh])
    didx = oracle.diff_arg_indices("hmlstm_update", 12)
    want = oracle.backward([wc.cpu().numpy(), wh.cpu().numpy()], o_parts, [host[j].shape for j in didx], threads=8)
    for k, (a, b) in enumerate(zip(got, want)):
        check_close(a.cpu().numpy(), b, f"node gradient {k}", rtol=1e-5, atol=2e-6)  # planes here are the oracle's own


def test_autograd_node_passes_torch_gradcheck_in_fp64():
    """torch's own numerical Jacobian check (central differences in fp64) on the node, for a
    function with a branch and broadcast arguments of every form, in all three storage modes; a
    gradient that is not asked for is not computed."""
    torch.manual_seed(5)
    dev = "cuda"
    A = torch.randn(6, 9, device=dev, dtype=torch.float64, requires_grad=True)
    Bm = (torch.rand(6, 9, device=dev, dtype=torch.float64) * 1.9 + 0.1).requires_grad_()
    r = torch.randn(9, device=dev, dtype=torch.float64, requires_grad=True)          # [9] -> [1 x 9]
    s = torch.randn(6, 1, device=dev, dtype=torch.float64, requires_grad=True)
    t = torch.randn((), device=dev, dtype=torch.float64, requires_grad=True)         # a 0-dim scalar
    for planes in ("all", "lean", "none"):
        fn = lambda *a: P.broadcast("branchy5", *a, planes=planes)
        assert torch.autograd.gradcheck(fn, (A, Bm, r, s, t), eps=1e-6, atol=1e-7, rtol=1e-6, nondet_tol=0.0)
        x = torch.randn(5, 7, device=dev, dtype=torch.float64, requires_grad=True)
        y = torch.randn(5, 7, device=dev, dtype=torch.float64, requires_grad=True)
        b = torch.randn(5, 1, device=dev, dtype=torch.float64, requires_grad=True)
        assert torch.autograd.gradcheck(lambda *a: P.broadcast("tanh_xy_b", *a, planes=planes), (x, y, b),
                                        eps=1e-6, atol=1e-7, rtol=1e-6, nondet_tol=0.0)
    out = P.broadcast("tanh_xy_b", x, y.detach(), b)
    gx, gb = torch.autograd.grad(out.sum(), [x, b])
    assert gx.shape == x.shape and gb.shape == b.shape


def _elementary_reference(xs):
    """(exp, log1p, sigma, tanh) and their derivatives at the points xs (exact binary values) in
    60-digit decimal arithmetic; entries where log1p is undefined (x <= -1) are None."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    one = Decimal(1)
    vals, ders = [], []
    for x in xs:
        d = Decimal(float(x))
        far = abs(d) > 2000  # beyond every floating-point range: the limits
        e = (Decimal("Infinity") if d > 0 else Decimal(0)) if far else d.exp()
        em = Decimal(0) if far else (-abs(d)).exp()
        q = Decimal(0) if far else (-2 * abs(d)).exp()
        sg = one / (one + em) if d >= 0 else em / (one + em)
        th = (one - q) / (one + q) * (1 if d >= 0 else -1)
        lg = (one + d).ln() if d > -1 else None
        if abs(d) < Decimal("1e-20"):  # 1 + d and 1 - q would round to 1 and 0 even at 60 digits: the series
            th = d - d ** 3 / 3 + 2 * d ** 5 / 15
            lg = d - d * d / 2 + d ** 3 / 3
        vals.append([e, lg, sg, th])
        ders.append([e, one / (one + d) if d > -1 else None, em / (one + em) ** 2, 4 * q / (one + q) ** 2])
    return vals, ders


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_elementary_functions_accuracy_in_ulps(dtype):
    """exp, log1p, sigma, tanh and their derivatives as the kernels compute them, over the whole
    range of the working precision -- saturation, tiny arguments, the neighbourhood of log1p's
    pole, results down to the smallest normal number -- against 60-digit values: every result is
    within a few units in the last place (far inside the tolerance of the parity tests, which
    only see arguments of order one)."""
    from decimal import Decimal
    f32 = dtype == np.float32
    big = 87.0 if f32 else 700.0
    # ... and on past the overflow of exp (fp32: 88.72, where 2^t is already inf while the correction
    # term may have either sign; fp64: 709.78): inf on both sides, never NaN
    beyond = np.linspace(big, 112.0 if f32 else 760.0, 251)
    pts = [np.linspace(-big, big, 801), np.linspace(-3, 3, 601), beyond, -beyond,
           np.concatenate([s * 10.0 ** np.arange(-30 if f32 else -200, 1, 1.5) for s in (1, -0.9)]),
           -1 + 10.0 ** -np.arange(1, 7 if f32 else 15), 10.0 ** np.arange(1, 30 if f32 else 200, 3.0)]
    xs = np.unique(np.concatenate(pts).astype(dtype))
    out_shape = (1, xs.size)
    dev = [to_dev(xs.reshape(out_shape))]
    fb = gpu_forward("elementary4", dev, want_branch=False)
    torch.cuda.synchronize()
    got_v = [o.cpu().numpy().reshape(-1) for o in fb.outs]
    got_d = [p.cpu().numpy().reshape(-1) for p in fb.partials]
    ref_v, ref_d = _elementary_reference(xs)
    info = np.finfo(dtype)
    names = ["exp", "log1p", "sigma", "tanh"]
    worst = {}
    for k, x in enumerate(xs):
        for which, got, ref in (("", got_v, ref_v), ("'", got_d, ref_d)):
            for i in range(4):
                r = ref[k][i]
                if r is None:
                    continue
                g = got[i][k]
                rf = float(r)
                if abs(rf) > info.max:       # overflows the working precision: inf on both sides
                    assert np.isinf(g) and (g > 0) == (rf > 0), (names[i] + which, float(x), g)
                    continue
                if abs(rf) < 8 * info.tiny:  # at the bottom of the range an intermediate is flushed to zero: no ulp bound
                    assert abs(float(g)) <= 16 * info.tiny, (names[i] + which, float(x), g)
                    continue
                ulp = Decimal(float(np.spacing(np.abs(dtype(rf)))))
                err = float(abs(Decimal(float(g)) - r) / ulp)
                key = names[i] + which
                if err > worst.get(key, (0.0, 0.0))[0]:
                    worst[key] = (err, float(x))
    print({k: (round(v[0], 2), v[1]) for k, v in worst.items()})
    limits = {"exp": 2.0, "exp'": 2.0, "log1p": 3.5, "log1p'": 2.0, "sigma": 3.0, "sigma'": 5.0, "tanh": 4.0, "tanh'": 6.0}
    for key, (err, x) in worst.items():
        assert err <= limits[key], f"{key}: {err:.2f} ulp at x = {x!r}"


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_division_accuracy_and_limits(dtype):
    """x1 / x2 and its partials 1 / x2, -x1 / x2^2 (second output of pair3 with x3 = 0) against exact
    rational arithmetic: a few units in the last place over twenty orders of magnitude, and the
    IEEE limits at x2 = +-0 and +-inf (inf and 0 with the right signs, never NaN)."""
    from fractions import Fraction
    rng = np.random.default_rng(12)
    mags = 10.0 ** np.arange(-10, 11, 0.5)
    x2 = np.concatenate([mags, -mags, rng.standard_normal(400)]).astype(dtype)
    x2 = x2[x2 != 0]
    x1 = (rng.standard_normal(x2.size) * 3).astype(dtype)
    x3 = np.zeros(x2.size, dtype)
    shape = (1, x2.size)
    fb = gpu_forward("pair3", [to_dev(a.reshape(shape)) for a in (x1, x2, x3)], want_branch=False)
    torch.cuda.synchronize()
    quot = fb.outs[1].cpu().numpy().reshape(-1)
    d1 = fb.partials[3].cpu().numpy().reshape(-1)   # plane index i * N_d + jd: output 1, argument 0
    d2 = fb.partials[4].cpu().numpy().reshape(-1)
    worst = [0.0, 0.0, 0.0]
    for k in range(x2.size):
        a, b = Fraction(float(x1[k])), Fraction(float(x2[k]))
        for n, (got, want) in enumerate(((quot[k], a / b), (d1[k], 1 / b), (d2[k], -a / (b * b)))):
            w = float(want)
            ulp = Fraction(float(np.spacing(np.abs(dtype(w)))))
            worst[n] = max(worst[n], float(abs(Fraction(float(got)) - want) / ulp))
    print("division, worst ulp:", [round(w, 2) for w in worst])
    assert worst[0] <= 2.5 and worst[1] <= 2.0 and worst[2] <= 4.0, worst
    # the limits
    x2 = np.array([0.0, -0.0, np.inf, -np.inf], dtype)
    x1 = np.array([2.0, 2.0, 2.0, 2.0], dtype)
    fb = gpu_forward("pair3", [to_dev(a.reshape(1, 4)) for a in (x1, x2, np.zeros(4, dtype))], want_branch=False)
    torch.cuda.synchronize()
    q = fb.outs[1].cpu().numpy().reshape(-1)
    inv = fb.partials[3].cpu().numpy().reshape(-1)
    assert q[0] == np.inf and q[1] == -np.inf and q[2] == 0 and q[3] == 0 and np.signbit(q[3]), q
    assert inv[0] == np.inf and inv[1] == -np.inf and inv[2] == 0 and inv[3] == 0, inv


def _same_with_specials(got, want, what):
    """NaN where the oracle has NaN, the same infinity where it has one, the usual tolerance elsewhere."""
    rt, at = TOL[want.dtype]
    g, w = got.astype(np.float64), want.astype(np.float64)
    bad = np.isnan(g) != np.isnan(w)
    bad |= np.isinf(w) & ~np.isnan(g) & (g != w)
    fin = np.isfinite(w) & ~np.isnan(g)
    with np.errstate(invalid="ignore"):
        bad |= fin & ~(np.abs(g - w) <= np.maximum(rt * np.abs(w), at))
    assert not bad.any(), f"{what}: {int(bad.sum())} elements; first at {tuple(np.argwhere(bad)[0])}: " \
                          f"got {got[tuple(np.argwhere(bad)[0])]} want {want[tuple(np.argwhere(bad)[0])]}"


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_special_values_propagate_as_in_the_oracle(dtype):
    """Infinities, NaN, signed zeros, arguments at the edge of exp's range and tiny ones, planted one
    argument at a time: values, partial planes and branch ids come out as the oracle's do (NaN for
    NaN, the same infinity, otherwise within tolerance), and so do gradients when adjoints and
    planes carry them."""
    specials = [np.inf, -np.inf, np.nan, 1e4, -1e4, 1e-30, -1e-30, 0.0, -0.0, 88.0, -88.0, 104.0, -104.0,
                89.0, -89.0, 95.0, -95.0, 101.0, -101.0, 110.0, -110.0]  # fp32 exp overflows from 88.73 on
    for op in ("tanh_xy_b", "branchy5", "hmlstm_update", "update_c", "elementary4"):
        R, C = 16, 4 * len(specials)
        args, adj = small_args(op, R, C, dtype, seed=3)
        control = {"hmlstm_update": (6, 7), "update_c": (4, 5)}.get(op, ())
        for j in range(len(args)):
            if j in control:
                continue
            planted = [a.copy() for a in args]
            tgt = planted[j]
            for k, sv in enumerate(specials):
                if tgt.shape[1] == 1:
                    tgt[k % tgt.shape[0], 0] = sv
                elif tgt.shape[0] == 1:
                    tgt[0, 4 * k:4 * k + 4] = sv
                else:
                    tgt[j % R, 4 * k:4 * k + 4] = sv
            fb = gpu_forward(op, [to_dev(a) for a in planted])
            torch.cuda.synchronize()
            with np.errstate(all="ignore"):
                o_out, o_parts, o_br = oracle.forward(op, planted, threads=4)
            assert np.array_equal(fb.branch.cpu().numpy(), o_br), (op, j)
            for i, (g, w) in enumerate(zip(fb.outs, o_out)):
                _same_with_specials(g.cpu().numpy(), w, f"{op}, special values in argument {j}, output {i}")
            for i, (g, w) in enumerate(zip(fb.partials, o_parts)):
                _same_with_specials(g.cpu().numpy(), w, f"{op}, special values in argument {j}, plane {i}")
    # backward: special values in an adjoint and in a plane reach exactly the gradients that sum over them
    args, adj = small_args("branchy5", 24, 260, dtype, seed=5)
    dev = [to_dev(a) for a in args]
    fb = gpu_forward("branchy5", dev)
    torch.cuda.synchronize()
    planes = [p.cpu().numpy() for p in fb.partials]
    adj[0][3, 7], adj[0][5, 100], adj[0][9, 200] = np.inf, np.nan, -np.inf
    planes[0][11, 30] = np.nan
    planes[2][13, 40] = np.inf
    shapes = [a.shape for a in args]
    bb = gpu_backward([to_dev(adj[0])], [to_dev(p) for p in planes], shapes)
    torch.cuda.synchronize()
    with np.errstate(all="ignore"):
        want = oracle.backward(adj, planes, shapes, threads=4)
    for k in range(5):
        _same_with_specials(bb.grads[k].cpu().numpy(), want[k], f"gradient {k} with special values")
    # an absent plane is a plane of zeros also for a non-finite adjoint (0 x inf is NaN): lean HM-LSTM layout
    op, args, adj = inputs.config_inputs(0, dtype=dtype)
    dev = [to_dev(a) for a in args]
    lean = P.alloc_forward(op, dev, lean=True).run(dev)
    adj[0][5, 3], adj[1][7, 2], adj[0][9, 9] = np.inf, np.nan, -np.inf
    didx = oracle.diff_arg_indices(op, 12)
    shapes = [args[j].shape for j in didx]
    adj_dev = [to_dev(a) for a in adj]
    gl = P.alloc_backward(adj_dev, lean.partials, shapes).run(adj_dev, lean.partials)
    torch.cuda.synchronize()
    with np.errstate(all="ignore"):
        want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in lean.partials], shapes, threads=4)
    for k in range(10):
        _same_with_specials(gl.grads[k].cpu().numpy(), want[k], f"lean layout, gradient {k} with special values")
    # the same call on the generic strided kernels (their reductions, too, form adjoint x 0 for an absent plane)
    generic = P.Options(force_generic=1)
    gg = P.alloc_backward(adj_dev, lean.partials, shapes, options=generic)
    assert P.bcast_dual_backward_plan(adj_dev, lean.partials, gg.grads, options=generic)["path"] == 2
    gg.run(adj_dev, lean.partials)
    torch.cuda.synchronize()
    for k in range(10):
        _same_with_specials(gg.grads[k].cpu().numpy(), want[k], f"lean layout on the generic kernels, gradient {k} with special values")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_cos_and_sin_accuracy_in_ulps(dtype):
    """cos x and its derivative -sin x (the Dual example of Sec. 2.2.1, op cos_x) against their
    power series in 60-digit arithmetic, over |x| <= 30 and down to tiny arguments: units in the
    last place, also next to the zeros of the functions."""
    from decimal import Decimal, getcontext
    getcontext().prec = 70
    one = Decimal(1)

    def series(x, first):  # sin (first = 1) or cos (first = 0)
        term = x if first else one
        total, k = term, first
        while abs(term) > Decimal("1e-75") or k < 4:
            k += 2
            term = -term * x * x / (k * (k - 1))
            total += term
        return total

    xs = np.unique(np.concatenate([np.linspace(-30, 30, 1201), 10.0 ** np.arange(-20, 0, 1.0), [np.pi / 2, np.pi, 3 * np.pi / 2]]).astype(dtype))
    fb = gpu_forward("cos_x", [to_dev(xs.reshape(1, -1))], want_branch=False)
    torch.cuda.synchronize()
    got = [fb.outs[0].cpu().numpy().reshape(-1), fb.partials[0].cpu().numpy().reshape(-1)]
    worst = [0.0, 0.0]
    for k, x in enumerate(xs):
        d = Decimal(float(x))
        for n, want in enumerate((series(d, 0), -series(d, 1))):
            ulp = Decimal(float(np.spacing(np.abs(dtype(float(want))))))
            worst[n] = max(worst[n], float(abs(Decimal(float(got[n][k])) - want) / ulp))
    print("cos, -sin worst ulp:", [round(w, 2) for w in worst])
    assert worst[0] <= 2.5 and worst[1] <= 2.5, worst


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_cancelling_sums_keep_their_small_terms(dtype):
    """Sums whose large terms cancel exactly and leave only small ones: products are formed
    without rounding and accumulated wide enough (double for fp32 data, double-double for fp64)
    that row sums, column sums and the full sum still come out right -- a plain sum in the
    working precision would return 0 for most of them."""
    rng = np.random.default_rng(77)
    R, C = 96, 2052
    big = dtype(2.0 ** 20 if dtype == np.float32 else 2.0 ** 58)
    P = rng.integers(-3, 4, (R, C)).astype(dtype)
    # +big / -big in 2 x 2 patterns (+ - / - +) scattered over the plane: every row and every column cancels
    for _ in range(1500):
        r1, r2 = rng.choice(R, 2, replace=False)
        c1, c2 = rng.choice(C, 2, replace=False)
        P[r1, c1] += big
        P[r1, c2] -= big
        P[r2, c1] -= big
        P[r2, c2] += big
    adj = np.full((R, C), 0.5, dtype)
    shapes = [(R, C), (R, 1), (1, C), (1, 1)]
    # one plane serves four gradients of the four classes (the planes of a call need not be distinct for reading)
    planes = [to_dev(P)] * 4
    bb = gpu_backward([to_dev(adj)], planes, shapes)
    torch.cuda.synchronize()
    want = oracle.backward([adj], [P] * 4, shapes, threads=8)
    exact_all = float(np.sum(adj.astype(np.longdouble) * P.astype(np.longdouble)))
    assert float(want[3].reshape(-1)[0]) == exact_all
    for k, what in enumerate(("elementwise", "row sums", "column sums", "full sum")):
        assert np.array_equal(bb.grads[k].cpu().numpy(), want[k]), what  # small integers and halves: exact on both sides


def test_expanded_adjoint_views():
    """An upstream adjoint that is itself a broadcast view (what reverse mode hands back from a
    sum: one value with strides 0, or a row expanded over the rows) gives the gradients of its
    materialised copy."""
    args, adj = small_args("branchy5", 37, 130, np.float32, seed=21)
    dev = [to_dev(a) for a in args]
    fb = gpu_forward("branchy5", dev)
    shapes = [a.shape for a in args]
    for view in (torch.full((1, 1), 0.75, device="cuda").expand(37, 130),
                 to_dev(adj[0][:1]).expand(37, 130),
                 to_dev(np.ascontiguousarray(adj[0][:, :1])).expand(37, 130)):
        assert not view.is_contiguous()
        got = gpu_backward([view], fb.partials, shapes)
        ref = gpu_backward([view.contiguous()], fb.partials, shapes)
        torch.cuda.synchronize()
        want = oracle.backward([view.cpu().numpy().copy()], [p.cpu().numpy() for p in fb.partials], shapes)
        for k in range(5):
            check_close(got.grads[k].cpu().numpy(), want[k], f"expanded adjoint, gradient {k}")
            check_close(ref.grads[k].cpu().numpy(), want[k], f"materialised adjoint, gradient {k}")


def test_row_expanded_planes_and_second_adjoint():
    """Read views that repeat one row (row stride 0 over many rows) among contiguous ones -- a plane, or
    an adjoint other than the first: the call must take kernels that address every view with its own row
    stride, and give the gradients of the materialised copies."""
    R, C = 300, 1100
    # M = 1: each plane of tanh(x*y + b) in turn as one row expanded over all rows
    args, adj = small_args("tanh_xy_b", R, C, np.float32, seed=31)
    dev = [to_dev(a) for a in args]
    fb = gpu_forward("tanh_xy_b", dev)
    shapes = [a.shape for a in args]
    adj_dev = [to_dev(adj[0])]
    for k in range(3):
        planes = list(fb.partials)
        planes[k] = fb.partials[k][7:8].expand(R, C)
        assert planes[k].stride() == (0, 1)
        bb = P.alloc_backward(adj_dev, planes, shapes)
        plan = P.bcast_dual_backward_plan(adj_dev, planes, bb.grads)
        assert plan["path"] == 2 or plan["uniform_stride"] == 0, plan
        bb.run(adj_dev, planes)
        torch.cuda.synchronize()
        want = oracle.backward(adj, [p.contiguous().cpu().numpy() for p in planes], shapes, threads=8)
        for j in range(3):
            check_close(bb.grads[j].cpu().numpy(), want[j], f"plane {k} row-expanded, gradient {j}")
    # M = 2: the second adjoint of pair3 as one row expanded over all rows (the first is the planner's sort key)
    args, adj = small_args("pair3", R, C, np.float64, seed=32)
    dev = [to_dev(a) for a in args]
    fb = gpu_forward("pair3", dev)
    shapes = [a.shape for a in args]
    a1 = to_dev(adj[1][:1]).expand(R, C)
    adj_dev = [to_dev(adj[0]), a1]
    bb = P.alloc_backward(adj_dev, fb.partials, shapes)
    plan = P.bcast_dual_backward_plan(adj_dev, fb.partials, bb.grads)
    assert plan["path"] == 2 or plan["uniform_stride"] == 0, plan
    bb.run(adj_dev, fb.partials)
    rb = P.alloc_recompute(fb.op_id, dev, adj_dev, shapes)
    assert P.bcast_dual_backward_recompute_plan(fb.op_id, dev, adj_dev, rb.grads)["uniform_stride"] == 0
    P.bcast_dual_backward_recompute(fb.op_id, dev, adj_dev, rb.grads, rb.workspace)
    torch.cuda.synchronize()
    want = oracle.backward([adj[0], a1.contiguous().cpu().numpy()], [p.cpu().numpy() for p in fb.partials], shapes, threads=8)
    for j in range(3):
        check_close(bb.grads[j].cpu().numpy(), want[j], f"second adjoint row-expanded, gradient {j}")
        check_close(rb.grads[j].cpu().numpy(), want[j], f"second adjoint row-expanded, recomputed gradient {j}")


@pytest.mark.parametrize("shape", [(200000, 3), (65536, 4), (300007, 1), (2, 600000), (1, 1000003)])
def test_tall_thin_and_long_flat_problems(shape):
    """Hundreds of thousands of rows of a few elements (256 rows per block step, column sums over
    all of them through many per-block partial sums) and the transposed extreme."""
    R, C = shape
    for op in ("branchy5", "hmlstm_update"):
        args, adj = small_args(op, R, C, np.float32, seed=R % 97)
        check_op(op, args, adj, threads=16, what=f"[{R} x {C}] ")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_rank3_problem_takes_vectors_along_the_innermost_dim(dtype):
    """An argument broadcast along the middle dim only keeps the problem at rank 3 (no two dims
    merge).  The tiled kernels take it as a batch of two-dim slices; the generic kernels (forced
    here) serve it with 16-byte accesses along the contiguous innermost dim where every view
    allows them and element by element where one does not."""
    generic = P.Options(force_generic=1)
    rng = np.random.default_rng(314)
    T_, B_, H_ = 6, 10, 64
    A = rng.standard_normal((T_, B_, H_)).astype(dtype)
    Bm = rng.uniform(0.1, 2, (T_, B_, H_)).astype(dtype)
    r = rng.standard_normal((T_, 1, H_)).astype(dtype)      # per step and feature, broadcast over the batch
    s = rng.standard_normal((1, B_, 1)).astype(dtype)
    t = rng.standard_normal((1, 1, 1)).astype(dtype)
    adj = [rng.standard_normal((T_, B_, H_)).astype(dtype)]
    dev = [to_dev(x) for x in (A, Bm, r, s, t)]
    fb = P.alloc_forward("branchy5", dev, want_branch=True)
    info = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, fb.branch)
    assert info["path"] == 1 and info["ndim"] == 3 and info["shape"] == [T_, B_, H_], info
    info = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, fb.branch, options=generic)
    assert info["path"] == 2 and info["ndim"] == 3 and info["vec"] == (4 if dtype == np.float32 else 2), info
    check_op("branchy5", [A, Bm, r, s, t], adj, what="rank 3 as slices ", recompute="required")
    check_op("branchy5", [A, Bm, r, s, t], adj, what="rank 3, generic, vectors ", options=generic)
    # an innermost extent that is not a multiple of the vector, and a view with padded rows whose
    # stride is not one either: element by element on the generic kernels
    A2, B2, r2, adj2 = A[..., :63], Bm[..., :63], r[..., :63], [adj[0][..., :63]]
    dev2 = [to_dev(x) for x in (A2, B2, r2, s, t)]
    f2 = P.alloc_forward("branchy5", dev2)
    assert P.bcast_dual_forward_plan(f2.op_id, dev2, f2.outs, f2.partials, options=generic)["vec"] == 1
    check_op("branchy5", [A2, B2, r2, s, t], adj2, what="rank 3 as slices, rows of 63 ", recompute="required")
    check_op("branchy5", [A2, B2, r2, s, t], adj2, what="rank 3, generic, elements ", options=generic)

    def padded(tn, k):  # rows padded by 3 elements: outer strides 67 and 670 keep no vector boundary
        if k != 0:
            return tn
        wide = torch.empty(T_, B_, H_ + 3, dtype=tn.dtype, device=tn.device)
        wide[..., :H_] = tn
        return wide[..., :H_]

    check_op("branchy5", [A, Bm, r, s, t], adj, view=padded, what="rank 3 as slices, one padded view ")
    check_op("branchy5", [A, Bm, r, s, t], adj, view=padded, what="rank 3, generic, one padded view ", options=generic)


def test_three_dim_benchmark_shape_at_full_size():
    """The three-dim workload bench.py times (`branchy5_3d_64x256x1024`: r broadcast along the middle dim only),
    every element of the values, planes, branch ids and gradients against the oracle, planes stored and recomputed."""
    args, adj = inputs.branchy5_3d_inputs(64, 256, 1024, seed=inputs.BASE_SEED + 500 + 64 + 256 + 1024)
    dev = [to_dev(a) for a in args]
    fb = P.alloc_forward("branchy5", dev)
    info = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials)
    assert info["path"] == 1 and info["ndim"] == 3, info
    del fb, dev
    check_op("branchy5", args, adj, threads=16, what="three dims at full size ", recompute="required")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_rank3_reductions_of_many_chunks(dtype):
    """Rank-3 problems with every kind of reduced gradient -- kept or summed along the outer dim,
    along rows, along columns: [T x 1 x H], [1 x B x 1], [1 x 1 x H], [T x 1 x 1], scalar -- on the
    tiled kernels (a batch of slices: one main launch and the second pass) and on the generic kernels,
    large enough that those cut their fibres into chunks (partial sums in the workspace, final
    kernel), in both lane arrangements."""
    generic = P.Options(force_generic=1)
    rng = np.random.default_rng(2718)
    T_, B_, H_ = 24, 70, 1030
    full = (T_, B_, H_)
    A = rng.standard_normal(full).astype(dtype)
    Bm = rng.uniform(0.1, 2, full).astype(dtype)
    adj = [rng.standard_normal(full).astype(dtype)]
    for rs, ss, ts in (((T_, 1, H_), (1, B_, 1), (1, 1, 1)), ((T_, 1, H_), (1, 1, H_), (T_, 1, 1))):
        r, s, t = (rng.standard_normal(sh).astype(dtype) for sh in (rs, ss, ts))
        dev = [to_dev(x) for x in (A, Bm, r, s, t)]
        fb = gpu_forward("branchy5", dev)
        shapes = [x.shape for x in (A, Bm, r, s, t)]
        grads = [torch.empty(sh, dtype=dev[0].dtype, device="cuda") for sh in shapes]
        adj_dev = [to_dev(adj[0])]
        info = P.bcast_dual_backward_plan(adj_dev, fb.partials, grads)
        assert info["path"] == 1 and info["ndim"] == 3 and info["n_launches"] == 2 and info["n_second_pass"] == 3, info
        info = P.bcast_dual_backward_plan(adj_dev, fb.partials, grads, options=generic)
        assert info["path"] == 2 and info["ndim"] == 3 and info["n_launches"] > 5  # some reductions need the final kernel
        assert P.bcast_dual_backward_workspace(adj_dev, fb.partials, grads, options=generic) > 0
        check_op("branchy5", [A, Bm, r, s, t], adj, threads=16, what=f"slices: r {rs} s {ss} t {ts} ", recompute="required")
        for steps in (1, 5):  # few and many partial sums per output for the second pass
            check_op("branchy5", [A, Bm, r, s, t], adj, threads=16, what=f"slices, {steps} row steps per block: r {rs} s {ss} t {ts} ",
                     options=P.Options(bwd_row_steps=steps), recompute=False)
        check_op("branchy5", [A, Bm, r, s, t], adj, threads=16, what=f"generic: r {rs} s {ss} t {ts} ", options=generic)
    # a gradient with the shape of a slice, summed over the slices only, stays with the generic kernels
    r, s, t = (rng.standard_normal(sh).astype(dtype) for sh in ((1, B_, H_), (1, B_, 1), (T_, 1, 1)))
    dev = [to_dev(x) for x in (A, Bm, r, s, t)]
    fb = gpu_forward("branchy5", dev)
    assert P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials)["path"] == 1
    grads = [torch.empty(x.shape, dtype=dev[0].dtype, device="cuda") for x in (A, Bm, r, s, t)]
    assert P.bcast_dual_backward_plan([to_dev(adj[0])], fb.partials, grads)["path"] == 2
    check_op("branchy5", [A, Bm, r, s, t], adj, threads=16, what="r [1 x B x H] ")


def _offset_by_one_element(t, k):
    """The same values in storage that starts one element past an aligned address (same strides)."""
    flat = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
    v = flat[1:].view(t.shape)
    v.copy_(t)
    return v


RAGGED_CASES = [("hmlstm_update", 3, 5), ("hmlstm_update", 33, 1023), ("hmlstm_update", 130, 1025), ("hmlstm_update", 9, 2051),
                ("branchy5", 7, 6), ("branchy5", 1, 4099), ("branchy5", 260, 259), ("pair3", 65, 1030), ("pair3", 2, 7),
                ("tanh_xy_b", 129, 4), ("update_c", 300, 1101), ("elementary4", 5, 777), ("linear12", 1000, 13),
                ("branchy5", 700, 4099), ("tanh_xy_b", 1500, 2049), ("tanh_xy_b", 300, 2047), ("tanh_xy_b", 100, 4095)]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_rows_the_vector_does_not_fit(dtype):
    """Rows whose length is not a multiple of the 16-byte vector, or that start off its boundary, go
    to the kernels that read unaligned vectors and finish each row element by element (forward,
    backward from planes, recompute): the plans say so, and everything matches the oracle -- the
    row's last columns, the sums over rows and columns that must not see anything past a row's end
    (pair3 divides: the lanes past the end evaluate it on zeros), the branch ids."""
    vec = 16 // np.dtype(dtype).itemsize
    for op, R, C in RAGGED_CASES:
        args, adj = small_args(op, R, C, dtype, seed=R + C)
        for view in (None, _offset_by_one_element):
            if view is None and C % vec == 0:
                continue  # aligned as it stands
            dev = [to_dev(a) for a in args]
            if view is not None:
                dev = [view(t, k) for k, t in enumerate(dev)]
            adj_dev = [to_dev(a) for a in adj]
            gshapes = [args[j].shape for j in oracle.diff_arg_indices(op, len(args))]
            fb = P.alloc_forward(op, dev)
            bb = P.alloc_backward(adj_dev, fb.partials, gshapes)
            rb = P.alloc_recompute(fb.op_id, dev, adj_dev, gshapes)
            plans = [P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials),
                     P.bcast_dual_backward_recompute_plan(fb.op_id, dev, adj_dev, rb.grads)]
            for plan in plans:
                assert plan["path"] == 1 and plan["vec"] == vec and plan["ragged"] == 1, (op, R, C, plan)
            # the planes and adjoints are aligned: only the row length sends this call there (and where
            # every gradient has the full shape the rows merge into one)
            plan = P.bcast_dual_backward_plan(adj_dev, fb.partials, bb.grads)
            assert plan["path"] == 1 and plan["vec"] == vec and plan["ragged"] == int(plan["shape"][-1] % vec != 0), (op, R, C, plan)
            if op == "hmlstm_update":  # the kernel compiled for this mix of gradient classes takes such rows too
                assert plan["specialized"] == 1
            if op == "tanh_xy_b" and -(-C // (256 * vec)) in (2, 4):  # ... and the one that finishes a row of 2 or 4 column chunks in one block
                assert plan["specialized"] == 1 and plan["n_launches"] == 1 and plan["grid_x"] == 1
            check_op(op, args, adj, view=view, what=f"[{R}x{C}{' off by one element' if view else ''}] ", recompute="required")


def test_rows_the_vector_does_not_fit_on_the_aligned_kernels():
    """With the option ragged_rows off such rows take the widest aligned access that fits (8 or 4 bytes)."""
    aligned = P.Options(ragged_rows=0)
    for dtype in DTYPES:
        for op, R, C in (("hmlstm_update", 33, 1023), ("hmlstm_update", 40, 1030), ("branchy5", 260, 259), ("pair3", 2, 7)):
            args, adj = small_args(op, R, C, dtype, seed=R + C)
            dev = [to_dev(a) for a in args]
            fb = P.alloc_forward(op, dev)
            plan = P.bcast_dual_forward_plan(fb.op_id, dev, fb.outs, fb.partials, options=aligned)
            widest = 16 // np.dtype(dtype).itemsize
            assert plan["ragged"] == 0 and (plan["vec"] < widest or C % widest == 0)
            check_op(op, args, adj, what=f"[{R}x{C} aligned accesses] ", recompute="required", options=aligned)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "f64"])
def test_lean_plane_layout_on_rows_of_odd_length(dtype):
    """Shared and absent planes on rows the vector does not fit: the kernel compiled for the lean
    mix takes them in its edge path; same gradients as with all planes, bit for bit, and as the oracle's."""
    op = "hmlstm_update"
    args, adj = small_args(op, 130, 1027, dtype, seed=77)
    dev, adj_dev = [to_dev(a) for a in args], [to_dev(a) for a in adj]
    shapes = [args[j].shape for j in oracle.diff_arg_indices(op, 12)]
    full = P.alloc_forward(op, dev).run(dev)
    lean = P.alloc_forward(op, dev, lean=True).run(dev)
    gf = P.alloc_backward(adj_dev, full.partials, shapes).run(adj_dev, full.partials)
    gl = P.alloc_backward(adj_dev, lean.partials, shapes).run(adj_dev, lean.partials)
    for plan in (P.bcast_dual_backward_plan(adj_dev, lean.partials, gl.grads), P.bcast_dual_backward_plan(adj_dev, full.partials, gf.grads)):
        assert plan["path"] == 1 and plan["ragged"] == 1 and plan["specialized"] == 1, plan
    torch.cuda.synchronize()
    for a, b in zip(gf.grads, gl.grads):
        assert torch.equal(a, b)
    want = oracle.backward(adj, [None if p is None else p.cpu().numpy() for p in lean.partials], shapes, threads=16)
    for k in range(10):
        check_close(gl.grads[k].cpu().numpy(), want[k], f"lean grad {k}")
