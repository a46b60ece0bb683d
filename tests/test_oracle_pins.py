"""CPU-only pins of the oracle: what the paper and the mathematics fix.

None of these tests touches the HIP path.  They are chosen so that a dropped
term, a wrong sign or index, a transposed plane or a wrong broadcast pairing in
oracle/bcast_oracle.c fails at least one of them.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import tape as T

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20181008)


# --------------------------------------------------------------------------- helpers
def shapes_for(op, R, C):
    """Full-rank argument shapes exercising full / row / column / scalar broadcasts."""
    full, row, col, sc = (R, C), (1, C), (R, 1), (1, 1)
    return {
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


def random_args(op, R, C, dtype=np.float64, rng=RNG):
    shp = shapes_for(op, R, C)
    args = [rng.standard_normal(s).astype(dtype) for s in shp]
    if op in ("hmlstm_update", "linear12"):
        args[6] = (rng.random(shp[6]) < 0.5).astype(dtype)
        args[7] = (rng.random(shp[7]) < 0.5).astype(dtype)
    if op == "update_c":
        args[4] = (rng.random(shp[4]) < 0.5).astype(dtype)
        args[5] = (rng.random(shp[5]) < 0.5).astype(dtype)
    if op == "pair3":
        args[1] = np.abs(args[1]) + 0.5  # the divisor stays away from 0
    if op == "elementary4":
        args[0] = (np.abs(args[0]) * 2 - 0.5).astype(dtype)  # log1p wants x > -1
    return args


def expand(a, shape):
    return np.broadcast_to(a, shape)


# tape programs: each op's formula re-expressed on tape variables ----------------
def tape_program(op, x):
    if op == "tanh_xy_b":
        return [T.tanh(x[0] * x[1] + x[2])]
    if op == "hmlstm_update":
        f, i, o, g, c, h, z, zb, bf, bi, bo, bg = x
        if z.v == 1.0:
            cn = T.sigmoid(i + bi) * T.tanh(g + bg)
        elif z.v == 0.0 and zb.v == 0.0:
            return [c * 1.0, h * 1.0]
        else:
            cn = T.sigmoid(f + bf) * c + T.sigmoid(i + bi) * T.tanh(g + bg)
        return [cn, T.sigmoid(o + bo) * T.tanh(cn)]
    if op == "linear12":
        f, i, o, g, c, h, z, zb, bf, bi, bo, bg = x
        return [f + i + o + g + c + h + bf + bi + bo + bg + z.v * zb.v,
                f * c + i * h + o * g + bf * bi + bo * bg]
    if op == "update_c":
        c, f, i, g, z1, z2 = x
        if z1.v == 1.0:
            return [T.sigmoid(i) * T.tanh(g)]
        if z1.v == 0.0 and z2.v == 0.0:
            return [c * 1.0]
        return [T.sigmoid(f) * c + T.sigmoid(i) * T.tanh(g)]
    if op == "branchy5":
        A, B, r, s, t = x
        if A.v + s.v > t.v:
            return [T.exp(-A) * B + r]
        return [T.log1p(A * A) * r - s]
    if op == "cos_x":
        return [T.cos(x[0])]
    if op == "elementary4":
        return [T.exp(x[0]), T.log1p(x[0]), T.sigmoid(x[0]), T.tanh(x[0])]
    if op == "scale_xt":
        return [x[0] * x[1]]
    if op == "pair3":
        return [x[0] * x[1] + T.sin(x[2]), x[0] / x[1] - x[2] * x[2]]
    if op == "prod_tanh":
        p = None
        for xi in x:
            t = T.tanh(xi if xi.v > 0.5 else -xi)
            p = t if p is None else p * t
        return [p]
    raise KeyError(op)


OPS = ["hmlstm_update", "tanh_xy_b", "branchy5", "update_c", "cos_x", "scale_xt", "pair3", "linear12", "elementary4"]


def assert_close(a, b, rtol, atol, what=""):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    err = np.abs(a - b)
    tol = np.maximum(rtol * np.abs(b), atol)
    assert np.all(err <= tol), f"{what}: max err {err.max():.3e} (worst tol ratio {(err / tol).max():.2f})"


# --------------------------------------------------------------------------- tape pin
@pytest.mark.parametrize("op", OPS)
def test_gradients_match_scalar_reverse_tape(op):
    """Whole chain forward -> planes -> backward against a reverse-mode tape run on the
    materialised expansion (Table 1; Sec. 2.2.3)."""
    R, C = 4, 5
    args = random_args(op, R, C)
    outs, parts, _ = oracle.forward(op, args)
    M = len(outs)
    adj = [RNG.standard_normal((R, C)) for _ in range(M)]
    didx = oracle.diff_arg_indices(op, len(args))
    grads = oracle.backward(adj, parts, [args[j].shape for j in didx])

    T.reset()
    leaves = [np.vectorize(T.Var, otypes=[object])(a) for a in args]
    total = T.Var(0.0)
    for r in range(R):
        for c in range(C):
            x = [expand(L, (R, C))[r, c] for L in leaves]
            ys = tape_program(op, x)
            for i in range(M):
                assert math.isclose(ys[i].v, outs[i][r, c], rel_tol=1e-13, abs_tol=1e-15)
                total = total + ys[i] * float(adj[i][r, c])
    T.backward(total)
    for k, j in enumerate(didx):
        want = np.vectorize(lambda v: v.adj)(leaves[j]).astype(np.float64)
        assert_close(grads[k], want, 1e-12, 1e-14, f"{op} grad of arg {j}")


@pytest.mark.parametrize("n", [1, 2, 5, 18])
def test_prod_tanh_against_tape(n):
    R, C = 3, 4
    args = [RNG.standard_normal((R, C)) + 0.5 for _ in range(n)]
    outs, parts, br = oracle.forward("prod_tanh", args)
    adj = [RNG.standard_normal((R, C))]
    grads = oracle.backward(adj, parts, [(R, C)] * n)
    for r in range(R):
        for c in range(C):
            T.reset()
            x = [T.Var(a[r, c]) for a in args]
            y = tape_program("prod_tanh", x)[0]
            T.backward(y)
            assert math.isclose(y.v, outs[0][r, c], rel_tol=1e-13)
            assert br[r, c] == sum(a[r, c] > 0.5 for a in args)
            for j in range(n):
                assert math.isclose(x[j].adj * adj[0][r, c], grads[j][r, c], rel_tol=1e-12, abs_tol=1e-15)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_prod_tanh_tie_takes_the_else_branch(dtype):
    """g(x) = x if x > 1/2 else -x (Sec. 3.4.1): exactly 1/2 is not greater than 1/2."""
    x = np.array([[0.5, np.nextafter(dtype(0.5), dtype(1.0)), 0.25]], dtype)
    outs, parts, br = oracle.forward("prod_tanh", [x])
    assert br.tolist() == [[0, 1, 0]]
    want = np.tanh(np.array([-0.5, float(x[0, 1]), -0.25]))
    np.testing.assert_allclose(outs[0][0], want.astype(dtype), rtol=2e-7 if dtype == np.float32 else 1e-15)
    assert parts[0][0, 0] < 0 < parts[0][0, 1]  # d tanh(-x)/dx < 0 on the else branch


# ----------------------------------------------------------------- finite differences
@pytest.mark.parametrize("op", OPS)
def test_partials_match_central_differences(op):
    """Stored planes are d y_i / d x_j of the branch taken (Sec. 2.2.2)."""
    R, C = 5, 6
    args = random_args(op, R, C)
    outs, parts, br = oracle.forward(op, args)
    didx = oracle.diff_arg_indices(op, len(args))
    Nd = len(didx)
    for k, j in enumerate(didx):
        h = 1e-6
        ap = [a.copy() for a in args]
        am = [a.copy() for a in args]
        ap[j] = ap[j] + h
        am[j] = am[j] - h
        yp, _, bp = oracle.forward(op, ap)
        ym, _, bm = oracle.forward(op, am)
        keep = (bp == br) & (bm == br)  # skip points within h of a predicate boundary
        assert keep.mean() > 0.9
        for i in range(len(outs)):
            fd = (yp[i] - ym[i]) / ((ap[j] - am[j]) * np.ones((R, C)))
            assert_close(parts[i * Nd + k][keep], fd[keep], 2e-7, 2e-8, f"{op} d y{i}/d x{j}")


# -------------------------------------------------------------------- structure pins
def test_eq1_broadcast_pairing_matches_paper_example():
    """b.(A, alpha, a): the n-vector pairs with the first dim, the scalar with all."""
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLDEN, "eq1_broadcast_example.txt"))
            if l.strip() and not l.startswith("#")]
    A = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    alpha = np.array([[10.0]])
    a = np.array([[0.25], [0.75]])
    outs, parts, _ = oracle.forward("pair3", [A, alpha, a])
    for (r, c, ar, ac, _al, ai) in rows:
        x1, x2, x3 = A[ar - 1, ac - 1], alpha[0, 0], a[ai - 1, 0]
        assert math.isclose(outs[0][r - 1, c - 1], x1 * x2 + math.sin(x3), rel_tol=1e-15)
        assert math.isclose(outs[1][r - 1, c - 1], x1 / x2 - x3 * x3, rel_tol=1e-15)


def test_jacobian_plane_order_matches_paper_expansion():
    order = [tuple(map(int, l.split())) for l in open(os.path.join(GOLDEN, "jacobian_plane_order.txt"))
             if l.strip() and not l.startswith("#")]
    x = [np.array([[1.5]]), np.array([[2.0]]), np.array([[0.3]])]
    _, parts, _ = oracle.forward("pair3", x)
    x1, x2, x3 = 1.5, 2.0, 0.3
    J = {(1, 1): x2, (1, 2): x1, (1, 3): math.cos(x3),
         (2, 1): 1 / x2, (2, 2): -x1 / x2 ** 2, (2, 3): -2 * x3}
    assert len(order) == len(parts) == 6
    for plane, i, j in order:
        assert math.isclose(parts[plane][0, 0], J[(i, j)], rel_tol=1e-15)


def test_cos_dual_example():
    """cos(Dual(x, y)) -> Dual(cos x, -sin x * y), Sec. 2.2.1, with unit seed."""
    x = np.linspace(-3, 3, 13).reshape(1, 13)
    outs, parts, _ = oracle.forward("cos_x", [x])
    assert_close(outs[0], np.cos(x), 1e-15, 1e-16)
    assert_close(parts[0], -np.sin(x), 1e-15, 1e-16)


@pytest.mark.parametrize("op", ["hmlstm_update", "branchy5", "tanh_xy_b"])
def test_jacobian_is_diagonal_per_element(op):
    """Perturbing one input element moves only the outputs it was expanded to (Sec. 2.2.2)."""
    R, C = 4, 5
    args = random_args(op, R, C)
    base, _, br0 = oracle.forward(op, args)
    didx = oracle.diff_arg_indices(op, len(args))
    for j in didx:
        a = args[j]
        for pos in [(0, 0), (a.shape[0] - 1, a.shape[1] - 1)]:
            pert = [x.copy() for x in args]
            pert[j][pos] += 1e-3
            new, _, _ = oracle.forward(op, pert)
            fibre = np.zeros((R, C), bool)
            fibre[(slice(None) if a.shape[0] == 1 else pos[0]),
                  (slice(None) if a.shape[1] == 1 else pos[1])] = True
            for i in range(len(base)):
                changed = new[i] != base[i]
                assert not np.any(changed & ~fibre), f"{op}: arg {j} leaked outside its fibre"


# ---------------------------------------------------------------- per-branch constants
def test_hmlstm_branch_constants():
    R, C = 8, 16
    args = random_args("hmlstm_update", R, C)
    # make sure all three branches appear: z, z_below per column
    args[6][0, :] = ([1, 0, 0, 1] * 4)
    args[7][0, :] = ([0, 0, 1, 1] * 4)
    outs, P, br = oracle.forward("hmlstm_update", args)
    Nd = 10  # f i o g c h b_f b_i b_o b_g
    F, I, O, G, Cc, H, BF, BI, BO, BG = range(10)
    c_, h_ = 0, 1
    pl = lambda i, j: P[i * Nd + j]
    z = np.broadcast_to(args[6], (R, C))
    zb = np.broadcast_to(args[7], (R, C))
    flush, copy = z == 1, (z == 0) & (zb == 0)
    upd = ~flush & ~copy
    assert np.array_equal(br, np.where(flush, 2, np.where(copy, 1, 0)))
    assert flush.any() and copy.any() and upd.any()
    # COPY: identity on c and h, everything else zero
    assert np.all(pl(c_, Cc)[copy] == 1) and np.all(pl(h_, H)[copy] == 1)
    assert np.array_equal(outs[0][copy], np.broadcast_to(args[4], (R, C))[copy])
    assert np.array_equal(outs[1][copy], np.broadcast_to(args[5], (R, C))[copy])
    for i in (c_, h_):
        for j in range(Nd):
            if (i, j) not in ((c_, Cc), (h_, H)):
                assert np.all(pl(i, j)[copy] == 0)
    # FLUSH: no dependence on c or f
    for i in (c_, h_):
        for j in (F, Cc, BF):
            assert np.all(pl(i, j)[flush] == 0)
    # UPDATE: d c'/d c = sigma(f + b_f) in (0, 1)
    sf = 1 / (1 + np.exp(-(args[0] + args[8])))
    assert_close(pl(c_, Cc)[upd], sf[upd], 1e-15, 0)
    # everywhere: c' ignores o and h; h' ignores h off COPY; bias planes equal gate planes
    for j in (O, H, BO):
        assert np.all(pl(c_, j) == 0)
    assert np.all(pl(h_, H)[~copy] == 0)
    for i in (c_, h_):
        for gate, bias in ((F, BF), (I, BI), (O, BO), (G, BG)):
            assert np.array_equal(pl(i, gate), pl(i, bias))


def test_hmlstm_closed_form_special_values():
    """sigma(ln 3) = 3/4, sigma(0) = 1/2, tanh(ln 2) = 3/5, applied to the cell update
    (Sec. 3.1 case equation); the pre-activations are split between gate and bias."""
    ln2, ln3 = math.log(2), math.log(3)
    c = (ln2 - 0.45) / 0.75  # makes c' = 3/4 c + 3/4 * 3/5 = ln 2 so tanh(c') = 3/5
    one = lambda v: np.array([[v]])
    base = dict(f=ln3 - 0.125, i=ln3 + 0.5, o=0.25, g=ln2 - 1.0, c=c, h=7.0,
                b_f=0.125, b_i=-0.5, b_o=-0.25, b_g=1.0)

    def run(z, zb):
        a = [one(base[k]) for k in ("f", "i", "o", "g", "c", "h")] + [one(z), one(zb)] + \
            [one(base[k]) for k in ("b_f", "b_i", "b_o", "b_g")]
        outs, P, br = oracle.forward("hmlstm_update", a)
        return [o[0, 0] for o in outs], [p[0, 0] for p in P], br[0, 0]

    # UPDATE (z = 0, z_below = 1)
    y, P, br = run(0.0, 1.0)
    assert br == 0
    dc = {"f": 3 / 4 * 1 / 4 * c, "i": 3 / 4 * 1 / 4 * 3 / 5, "g": 3 / 4 * (1 - 9 / 25), "c": 3 / 4}
    want_c = [dc["f"], dc["i"], 0, dc["g"], dc["c"], 0, dc["f"], dc["i"], 0, dc["g"]]
    k = 1 / 2 * (1 - 9 / 25)  # sigma(o) (1 - tanh^2 c')
    dho = 1 / 2 * 1 / 2 * 3 / 5
    want_h = [k * dc["f"], k * dc["i"], dho, k * dc["g"], k * dc["c"], 0, k * dc["f"], k * dc["i"], dho, k * dc["g"]]
    assert_close(y, [ln2, 0.3], 1e-14, 0)
    assert_close(P, want_c + want_h, 1e-13, 1e-16)
    # FLUSH (z = 1): c' = 3/4 * 3/5 = 9/20
    y, P, br = run(1.0, 0.0)
    assert br == 2
    tau = math.tanh(0.45)
    assert_close(y, [0.45, 0.5 * tau], 1e-14, 0)
    k = 0.5 * (1 - tau * tau)
    want_c = [0, dc["i"], 0, dc["g"], 0, 0, 0, dc["i"], 0, dc["g"]]
    dho = 0.25 * tau
    want_h = [0, k * dc["i"], dho, k * dc["g"], 0, 0, 0, k * dc["i"], dho, k * dc["g"]]
    assert_close(P, want_c + want_h, 1e-13, 1e-16)
    # COPY (z = 0, z_below = 0)
    y, P, br = run(0.0, 0.0)
    assert br == 1 and y == [c, 7.0]
    want = [0.0] * 20
    want[4] = 1.0
    want[10 + 5] = 1.0
    assert P == want
    # off-grid control values fall to UPDATE
    assert run(0.5, 0.0)[2] == 0 and run(float("nan"), 0.0)[2] == 0 and run(0.0, 2.0)[2] == 0


def test_update_c_is_hmlstm_cell_without_bias():
    """The paper's six-argument fused update (Sec. 3.2.3) equals the c' output of the
    biased cell with zero biases."""
    R, C = 6, 7
    a = random_args("hmlstm_update", R, C)
    for k in range(8, 12):
        a[k][...] = 0
    o1, P1, b1 = oracle.forward("hmlstm_update", a)
    o2, P2, b2 = oracle.forward("update_c", [a[4], a[0], a[1], a[3], a[6], a[7]])
    assert np.array_equal(b1, b2) and np.array_equal(o1[0], o2[0])
    for mine, theirs in ((0, 4), (1, 0), (2, 1), (3, 3)):  # c f i g  <-  planes of c'
        assert np.array_equal(P2[mine], P1[theirs])


def test_branchy5_branch_constants_and_predicate_precision():
    R, C = 16, 16
    args = random_args("branchy5", R, C)
    outs, P, br = oracle.forward("branchy5", args)
    A, B, r, s, t = [np.broadcast_to(a, (R, C)) for a in args]
    assert np.array_equal(br, (A + s > t).astype(np.uint8))
    tr = br == 1
    assert tr.any() and (~tr).any()
    assert np.all(P[2][tr] == 1) and np.all(P[3][tr] == 0) and np.all(P[1][~tr] == 0)
    assert np.all(P[3][~tr] == -1) and np.all(P[4] == 0)
    assert_close(P[1][tr], np.exp(-A)[tr], 1e-15, 0)
    assert_close(P[2][~tr], np.log1p(A * A)[~tr], 1e-15, 0)
    # fp32 variant: the sum is rounded to float before the compare, and ties go to "else"
    A32 = np.array([[1.0, 1.0, 3.0]], np.float32)
    s32 = np.array([[2.0 ** -25]], np.float32)      # A + s rounds back to A in float
    t32 = np.array([[1.0]], np.float32)
    _, _, b32 = oracle.forward("branchy5", [A32, np.ones_like(A32), np.ones_like(A32), s32, t32])
    assert b32.tolist() == [[0, 0, 1]]
    _, _, b64 = oracle.forward("branchy5", [A32.astype(np.float64), np.ones((1, 3)), np.ones((1, 3)),
                                            s32.astype(np.float64), t32.astype(np.float64)])
    assert b64.tolist() == [[1, 1, 1]]
    # exact ties in fp64 also take the else branch (strict >); just above the tie takes the other
    A64 = np.array([[0.5, 0.5 + 2.0 ** -52]], np.float64)
    _, _, bt = oracle.forward("branchy5", [A64, np.ones((1, 2)), np.ones((1, 2)), np.array([[0.5]]), np.array([[1.0]])])
    assert bt.tolist() == [[0, 1]]


def test_branchy5_closed_form_values():
    """exp(-ln 2) = 1/2 ; log1p(e - 1) = 1."""
    one = lambda v: np.array([[v]])
    A = math.log(2)
    y, P, br = oracle.forward("branchy5", [one(A), one(3.0), one(0.25), one(1.0), one(0.0)])
    assert br[0, 0] == 1
    assert_close([y[0][0, 0]] + [p[0, 0] for p in P], [1.75, -1.5, 0.5, 1, 0, 0], 1e-15, 0)
    A = -math.sqrt(math.e - 1)
    y, P, br = oracle.forward("branchy5", [one(A), one(3.0), one(0.25), one(1.0), one(5.0)])
    assert br[0, 0] == 0
    assert_close([y[0][0, 0]] + [p[0, 0] for p in P],
                 [0.25 - 1.0, 2 * A * 0.25 / math.e, 0, 1.0, -1, 0], 1e-14, 0)


# ---------------------------------------------------------------------- reduction rule
def test_no_broadcast_means_elementwise_product():
    """Table 1, full-shape argument: grad = adj .* partial, exactly."""
    adj = [RNG.standard_normal((5, 7)).astype(np.float32)]
    P = [RNG.standard_normal((5, 7)).astype(np.float32)]
    g = oracle.backward(adj, P, [(5, 7)])[0]
    assert np.array_equal(g, (adj[0].astype(np.float64) * P[0]).astype(np.float32))


def test_ones_count_expanded_elements():
    """adjoint = 1 and partial = 1: gradient = number of elements the argument was copied to."""
    R, C = 6, 9
    ones = np.ones((R, C))
    for shape, count in (((R, C), 1), ((1, C), R), ((R, 1), C), ((1, 1), R * C)):
        g = oracle.backward([ones], [ones], [shape])[0]
        assert g.shape == shape and np.all(g == count)


def test_sums_are_exact_on_cancelling_data():
    """Sum over expanded dims against exact rational arithmetic; data chosen to cancel."""
    R, C = 7, 33
    adj = [RNG.standard_normal((R, C)).astype(np.float32) * np.float32(1e4) for _ in range(2)]
    P = [RNG.standard_normal((R, C)).astype(np.float32) for _ in range(2)]
    P[0][:, -1] = 0
    adj[0][:, -1] = 1
    # last column cancels the rest of output 0's row sum to ~0
    for r in range(R):
        tot = sum(Fraction(float(adj[0][r, c])) * Fraction(float(P[0][r, c])) for c in range(C - 1))
        P[0][r, -1] = np.float32(-float(tot))
    shapes = [(R, 1)]
    g = oracle.backward(adj, P, shapes)[0]
    for r in range(R):
        exact = sum(Fraction(float(adj[i][r, c])) * Fraction(float(P[i][r, c]))
                    for i in range(2) for c in range(C))
        assert g[r, 0] == np.float32(float(exact))
    # column sums and the full sum, M = 2, fp64
    adj64 = [a.astype(np.float64) for a in adj]
    P64 = [p.astype(np.float64) for p in P]
    gc, gs = oracle.backward(adj64 + [], P64[:1] + P64[:1] + P64[1:] + P64[1:], [(1, C), (1, 1)])
    for c in range(C):
        exact = sum(Fraction(float(adj64[0][r, c])) * Fraction(float(P64[0][r, c])) +
                    Fraction(float(adj64[1][r, c])) * Fraction(float(P64[1][r, c])) for r in range(R))
        assert gc[0, c] == float(exact)
    exact = sum(Fraction(float(adj64[i][r, c])) * Fraction(float(P64[i][r, c]))
                for i in range(2) for r in range(R) for c in range(C))
    assert gs[0, 0] == float(exact)
    # terms whose partial sums need more bits than any machine format has: 2^70 + 40 ones - 2^70
    # is 40; a sum that merely runs in a wide format answers 0
    n = 40
    a = np.ones((1, n + 2), np.float64)
    q = np.ones((1, n + 2), np.float64)
    a[0, 0], q[0, 0] = 2.0 ** 35, 2.0 ** 35
    a[0, -1], q[0, -1] = -(2.0 ** 35), 2.0 ** 35
    assert oracle.backward([a], [q], [(1, 1)])[0][0, 0] == float(n)
    assert oracle.backward([a.T.copy()], [q.T.copy()], [(1, 1)])[0][0, 0] == float(n)


def test_plane_order_is_output_major_in_backward():
    """grad_j uses planes [i*N_d + j]: swapping to argument-major must change the result."""
    R, C = 3, 4
    adj = [RNG.standard_normal((R, C)) for _ in range(2)]
    P = [RNG.standard_normal((R, C)) for _ in range(6)]  # M = 2, N_d = 3
    g = oracle.backward(adj, P, [(R, C)] * 3)
    for j in range(3):
        assert_close(g[j], adj[0] * P[j] + adj[1] * P[3 + j], 1e-15, 1e-17)
    g = oracle.backward(adj, [P[0], None, P[2], None, P[4], P[5]], [(R, C)] * 3)
    assert_close(g[0], adj[0] * P[0], 1e-15, 1e-17)
    assert_close(g[1], adj[1] * P[4], 1e-15, 1e-17)


def test_hmlstm_bias_gradient_is_row_sum_of_gate_gradient():
    R, C = 9, 21
    args = random_args("hmlstm_update", R, C)
    outs, P, _ = oracle.forward("hmlstm_update", args)
    adj = [RNG.standard_normal((R, C)) for _ in range(2)]
    didx = oracle.diff_arg_indices("hmlstm_update", 12)
    assert didx == [0, 1, 2, 3, 4, 5, 8, 9, 10, 11]
    g = oracle.backward(adj, P, [args[j].shape for j in didx])
    for gate, bias in ((0, 6), (1, 7), (2, 8), (3, 9)):
        assert g[bias].shape == (R, 1)
        assert_close(g[bias][:, 0], g[gate].sum(axis=1), 1e-13, 1e-14)


def test_branchy5_scalar_gradient_is_zero():
    args = random_args("branchy5", 8, 8)
    _, P, _ = oracle.forward("branchy5", args)
    g = oracle.backward([np.ones((8, 8))], P, [a.shape for a in args])
    assert g[4].shape == (1, 1) and g[4][0, 0] == 0.0


def test_rank3_and_rank1_shapes():
    """The definition holds for any rank (Sec. 2.1.1): compare with numpy broadcasting."""
    x = RNG.standard_normal((3, 1, 5))
    t = RNG.standard_normal((1, 4, 1))
    outs, P, _ = oracle.forward("scale_xt", [x, t])
    assert outs[0].shape == (3, 4, 5)
    assert_close(outs[0], x * t, 1e-15, 0)
    adj = [RNG.standard_normal((3, 4, 5))]
    gx, gt = oracle.backward(adj, P, [x.shape, t.shape])
    assert_close(gx, (adj[0] * t).sum(axis=1, keepdims=True), 1e-14, 1e-15)
    assert_close(gt, (adj[0] * x).sum(axis=(0, 2), keepdims=True), 1e-14, 1e-15)
    v = RNG.standard_normal((11,))
    outs, P, _ = oracle.forward("cos_x", [v])
    assert outs[0].shape == (11,)


def test_middle_dim_broadcast_equals_the_same_problem_with_materialised_arguments():
    """The three-dim benchmark shape (r broadcast along the middle dim only, s along the two others, Sec. 2.1.1):
    the oracle's values and planes equal those of the same call with r and s expanded to the full shape by
    numpy, and the reduced gradients are the sums of the expanded call's gradients over the broadcast dims."""
    from paper_1810_08297_amd import inputs
    args, adj = inputs.branchy5_3d_inputs(3, 5, 7, seed=11, dtype=np.float64)
    assert [a.shape for a in args] == [(3, 5, 7), (3, 5, 7), (3, 1, 7), (1, 5, 1), (1, 1, 1)] and adj[0].shape == (3, 5, 7)
    margs, _ = inputs.branchy5_3d_inputs(3, 5, 7, seed=11, dtype=np.float64, merging=True)
    assert [a.shape for a in margs] == [(3, 5, 7), (3, 5, 7), (1, 1, 7), (3, 5, 1), (1, 1, 1)]
    full = [np.ascontiguousarray(np.broadcast_to(a, (3, 5, 7))) for a in args]
    outs, P, br = oracle.forward("branchy5", args)
    outs_f, P_f, br_f = oracle.forward("branchy5", full)
    assert np.array_equal(outs[0], outs_f[0]) and np.array_equal(br, br_f)
    assert all(np.array_equal(a, b) for a, b in zip(P, P_f))
    g = oracle.backward(adj, P, [a.shape for a in args])
    g_f = oracle.backward(adj, P_f, [a.shape for a in full])
    assert np.array_equal(g[0], g_f[0]) and np.array_equal(g[1], g_f[1])
    assert_close(g[2], g_f[2].sum(axis=1, keepdims=True), 1e-14, 1e-15)
    assert_close(g[3], g_f[3].sum(axis=(0, 2), keepdims=True), 1e-14, 1e-15)
    assert_close(g[4], g_f[4].sum(keepdims=True), 1e-14, 1e-15)


def test_fp32_outputs_are_correctly_rounded_from_wide_evaluation():
    args = random_args("tanh_xy_b", 6, 6, np.float32)
    o32, P32, _ = oracle.forward("tanh_xy_b", args)
    o64, P64, _ = oracle.forward("tanh_xy_b", [a.astype(np.float64) for a in args])
    assert o32[0].dtype == np.float32
    assert np.array_equal(o32[0], o64[0].astype(np.float32))
    for a, b in zip(P32, P64):
        assert np.array_equal(a, b.astype(np.float32))


def test_errors():
    with pytest.raises(KeyError):
        oracle.forward("nope", [np.zeros((1, 1))])
    with pytest.raises(ValueError):
        oracle.forward("tanh_xy_b", [np.zeros((2, 2)), np.zeros((2, 2))])
    with pytest.raises(ValueError):
        oracle.forward("tanh_xy_b", [np.zeros((2, 3)), np.zeros((2, 2)), np.zeros((2, 1))])


@pytest.mark.parametrize("op", ["hmlstm_update", "update_c", "tanh_xy_b", "branchy5"])
def test_gradients_match_library_reverse_mode_on_select_form(op):
    """A third, independent differentiator: the same functions written as whole-array library
    primitives with both branches computed and selected (no scalar `if`), differentiated by
    torch.autograd in fp64 on the CPU.  Agreement says the branch handling, the broadcast
    reduction and every closed-form partial of the oracle are what plain reverse mode gives."""
    import torch
    from select_form import values_and_gradients
    rng = np.random.default_rng(77)
    R, C = 23, 41
    full, row, col, sc = (R, C), (1, C), (R, 1), (1, 1)
    shp = {"hmlstm_update": [full] * 6 + [row, row] + [col] * 4, "update_c": [full] * 4 + [row, row],
           "tanh_xy_b": [full, full, col], "branchy5": [full, full, row, col, sc]}[op]
    args = [rng.standard_normal(s) for s in shp]
    for k in {"hmlstm_update": (6, 7), "update_c": (4, 5)}.get(op, ()):
        args[k] = (rng.random(shp[k]) < 0.5).astype(np.float64)
    n_out = oracle.op_info(op)[1]
    adj = [rng.standard_normal(full) for _ in range(n_out)]
    o_out, o_parts, _ = oracle.forward(op, args, threads=2)
    didx = oracle.diff_arg_indices(op, len(args))
    want = oracle.backward(adj, o_parts, [args[j].shape for j in didx], threads=2)
    outs, grads = values_and_gradients(op, [torch.from_numpy(a) for a in args], [torch.from_numpy(a) for a in adj])
    for g, w in zip(outs, o_out):
        np.testing.assert_allclose(g.detach().numpy(), w, rtol=1e-13, atol=1e-14)
    for g, w in zip(grads, want):
        np.testing.assert_allclose(g.numpy().reshape(w.shape), w, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------- 60-digit arithmetic
def _dec_values():
    """The ops' VALUES only, written out in decimal arithmetic of 60 digits (Python's decimal
    module: its exp and ln are correctly rounded at the context's precision).  `ctl` holds the
    unperturbed arguments: predicates read those (Sec. 2.2.1: a comparison of dual numbers
    compares the value parts), so that a perturbed evaluation stays on the branch of the point."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    one = Decimal(1)
    sig = lambda x: one / (one + (-x).exp())
    tanh = lambda x: (one - (-2 * x).exp()) / (one + (-2 * x).exp())

    def tanh_xy_b(a, ctl):
        x, y, b = a
        return [tanh(x * y + b)]

    def branchy5(a, ctl):
        A, B, r, s, t = a
        if ctl[0] + ctl[3] > ctl[4]:
            return [(-A).exp() * B + r]
        return [(one + A * A).ln() * r - s]

    def hmlstm_update(a, ctl):
        f, i, o, g, c, h, z, zb, bf, bi, bo, bg = a
        if ctl[6] == 1:                        # FLUSH
            cn = sig(i + bi) * tanh(g + bg)
        elif ctl[6] == 0 and ctl[7] == 0:      # COPY
            return [c, h]
        else:                                  # UPDATE
            cn = sig(f + bf) * c + sig(i + bi) * tanh(g + bg)
        return [cn, sig(o + bo) * tanh(cn)]

    def update_c(a, ctl):  # the paper's cell update, Sec. 3.2.3: arguments c f i g z1 z2
        c, f, i, g, z1, z2 = a
        if ctl[4] == 1:
            return [sig(i) * tanh(g)]
        if ctl[4] == 0 and ctl[5] == 0:
            return [c]
        return [sig(f) * c + sig(i) * tanh(g)]

    def series(x, first):  # sin (first = 1) or cos (first = 0) by their power series, |x| < 8
        term = x if first else one
        total, k = term, first
        while abs(term) > Decimal("1e-70"):
            k += 2
            term = -term * x * x / (k * (k - 1))
            total += term
        return total

    def cos_x(a, ctl):
        return [series(a[0], 0)]

    def elementary4(a, ctl):
        return [a[0].exp(), (one + a[0]).ln(), sig(a[0]), tanh(a[0])]

    def scale_xt(a, ctl):
        return [a[0] * a[1]]

    def pair3(a, ctl):
        return [a[0] * a[1] + series(a[2], 1), a[0] / a[1] - a[2] * a[2]]

    def prod_tanh(a, ctl):  # Sec. 3.4.1
        p = one
        for x, x0 in zip(a, ctl):
            p *= tanh(x if x0 > Decimal("0.5") else -x)
        return [p]

    return {"tanh_xy_b": (tanh_xy_b, ()), "branchy5": (branchy5, ()), "hmlstm_update": (hmlstm_update, (6, 7)),
            "update_c": (update_c, (4, 5)), "cos_x": (cos_x, ()), "elementary4": (elementary4, ()), "scale_xt": (scale_xt, ()), "pair3": (pair3, ()),
            "prod_tanh": (prod_tanh, ())}


@pytest.mark.parametrize("op", ["tanh_xy_b", "branchy5", "hmlstm_update", "update_c", "cos_x", "scale_xt", "pair3", "prod_tanh", "elementary4"])
def test_fp64_outputs_match_sixty_digit_values_and_their_difference_quotients(op):
    """Every value the oracle returns in fp64 is the 60-digit value rounded to fp64, and every
    partial is the 60-digit central difference quotient of the value function (step 1e-25: the
    quotient is the derivative to some 45 digits), both to within one unit in the last place (two
    for the ops that call sin and cos).  The derivative formulas of the oracle appear nowhere in
    this test."""
    from decimal import Decimal
    value_fn, control = _dec_values()[op]
    rng = np.random.default_rng(606)
    R, C = 5, 7
    if op == "prod_tanh":
        args = [rng.standard_normal((R, C)) + 0.5 for _ in range(4)]
    else:
        args = random_args(op, R, C, np.float64, rng)
    outs, parts, _ = oracle.forward(op, args)
    M = len(outs)
    diff = [j for j in range(len(args)) if j not in control]
    nd = len(diff)
    assert len(parts) == M * nd
    h = Decimal("1e-25")
    ulp, tiny = Decimal("4.5e-16") if op in ("cos_x", "pair3") else Decimal("2.3e-16"), Decimal("1e-300")
    for r in range(R):
        for c in range(C):
            x = [Decimal(float(np.broadcast_to(a, (R, C))[r, c])) for a in args]
            vals = value_fn(x, x)
            for i in range(M):
                assert abs(Decimal(float(outs[i][r, c])) - vals[i]) <= max(abs(vals[i]) * ulp, tiny), (op, r, c, i)
            for jd, j in enumerate(diff):
                up, dn = list(x), list(x)
                up[j] += h
                dn[j] -= h
                vu, vd = value_fn(up, x), value_fn(dn, x)
                for i in range(M):
                    want = (vu[i] - vd[i]) / (2 * h)
                    got = Decimal(float(parts[i * nd + jd][r, c]))
                    assert abs(got - want) <= max(abs(want) * ulp, Decimal("1e-40")), (op, r, c, i, j, float(got), str(want))


def test_sums_with_infinite_and_nan_terms_follow_ieee():
    """Table 1's sum of products with non-finite terms: one infinity among finite terms gives that
    infinity, opposite infinities or a NaN term give NaN, 0 x inf is NaN, and rows without such
    terms are untouched (the compensation of the summation must not turn inf into NaN)."""
    R, C = 5, 8
    adj = [np.ones((R, C))]
    P = [np.full((R, C), 0.25)]
    P[0][0, 3] = np.inf                     # row 0: one +inf
    P[0][1, 2], P[0][1, 6] = np.inf, -np.inf  # row 1: both
    P[0][2, 5] = np.nan                     # row 2: NaN
    adj[0][3, 1], P[0][3, 1] = 0.0, np.inf  # row 3: 0 x inf
    with np.errstate(all="ignore"):
        rows = oracle.backward(adj, P, [(R, 1)])[0].reshape(-1)
        full = oracle.backward(adj, P, [(R, C)])[0]
        cols = oracle.backward(adj, P, [(1, C)])[0].reshape(-1)
    assert rows[0] == np.inf and np.isnan(rows[1]) and np.isnan(rows[2]) and np.isnan(rows[3]) and rows[4] == 2.0
    assert full[0, 3] == np.inf and full[1, 6] == -np.inf and np.isnan(full[2, 5]) and np.isnan(full[3, 1]) and full[4, 0] == 0.25
    assert cols[3] == np.inf and cols[2] == np.inf and cols[6] == -np.inf and np.isnan(cols[5]) and np.isnan(cols[1])
    assert cols[0] == 1.25 and cols[7] == 1.25


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_absent_plane_is_a_plane_of_zeros_also_for_nonfinite_adjoints(dtype):
    """Table 1's product adjoint x partial with a plane the caller did not store (None): the plane
    counts as zeros IN EVERY RESPECT, so a call with None and the same call with an explicit plane of
    zeros give the same bits -- also where the adjoint is infinite or NaN (inf x 0 = NaN, not "no
    term") -- for full-shape, row-sum, column-sum and all-sum gradients.  A backward that skipped
    absent planes would return 0 or the other outputs' finite sum there."""
    rng = np.random.default_rng(5)
    R, C = 6, 7
    shapes = [(R, C), (R, 1), (1, C), (1, 1)]
    for M in (1, 2):
        adj = [rng.standard_normal((R, C)).astype(dtype) for _ in range(M)]
        adj[0][1, 2] = np.inf
        adj[0][3, 4] = -np.inf
        adj[0][4, 0] = np.nan
        if M == 2:
            adj[1][2, 5] = np.inf
        nd = len(shapes)
        planes = [rng.standard_normal((R, C)).astype(dtype) for _ in range(M * nd)]
        for absent_output in range(M):
            with_none = list(planes)
            with_zero = list(planes)
            for jd in range(nd):
                with_none[absent_output * nd + jd] = None
                with_zero[absent_output * nd + jd] = np.zeros((R, C), dtype)
            with np.errstate(all="ignore"):
                a = oracle.backward(adj, with_none, shapes)
                b = oracle.backward(adj, with_zero, shapes)
            for ga, gb, shp in zip(a, b, shapes):
                assert np.array_equal(ga.view(np.uint32 if dtype == np.float32 else np.uint64),
                                      gb.view(np.uint32 if dtype == np.float32 else np.uint64)), (M, absent_output, shp)
            full, rows, cols, tot = a
            if absent_output == 0:  # the absent planes meet the non-finite adjoints of output 0
                assert np.isnan(full[1, 2]) and np.isnan(full[3, 4]) and np.isnan(full[4, 0])
                assert np.isnan(rows[1, 0]) and np.isnan(rows[3, 0]) and np.isnan(rows[4, 0]) and np.isfinite(rows[0, 0])
                assert np.isnan(cols[0, 2]) and np.isnan(cols[0, 4]) and np.isnan(cols[0, 0]) and np.isfinite(cols[0, 1])
                assert np.isnan(tot[0, 0])
                assert np.isfinite(full[0, 0]) and (M == 1 or np.isfinite(rows[5, 0]))
            else:  # output 1's planes are absent: its one infinite adjoint, at (2, 5), gives NaN there
                assert np.isnan(full[2, 5]) and np.isnan(rows[2, 0]) and np.isnan(cols[0, 5]) and np.isnan(tot[0, 0])
