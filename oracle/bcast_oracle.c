/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of mixed-mode differentiation
 * of a broadcast (arXiv 1810.08297): it exists so that the HIP path can be
 * checked against something that shares no code with it.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the product never does.
 *
 * What it computes
 *   forward : for every element e of the unified output shape (Sec. 2.1.1), fetch
 *             each argument with broadcast indexing (size-1 dim -> index 0), evaluate
 *             b directly, and evaluate the analytic partials d y_i / d x_j of the
 *             branch taken at that element -- the diagonal of the broadcast Jacobian
 *             (Sec. 2.2.2, the broadcast-Jacobian observation).
 *   backward: grad_j[a] = sum over the elements e that argument element a was
 *             expanded to, of sum_i adj_i[e] * P_ij[e]  (Table 1: a broadcast argument
 *             gets the dot product, a full-shape argument the elementwise product).
 *
 * Arithmetic: values and partials are evaluated in long double (x87 80-bit, 64-bit
 * significand) from the exactly-converted inputs and rounded once to the storage
 * type.  Predicates are evaluated in the WORKING precision (float for the fp32
 * variant, double for fp64) exactly as written (A + s > t, never A > t - s), so
 * branch ids have one correct value.  Sums use Neumaier-compensated long double.
 *
 * Pins (tests, CPU only): central finite differences, a scalar reverse-mode tape on
 * the materialised expansion, the diagonal-Jacobian and sum-over-expanded-dims
 * invariants, per-branch constants, the paper's b.(A, alpha, a) indexing example,
 * closed-form special values, exact rational sums.  Every function below is pinned.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -ffp-contract=off -fexcess-precision=standard
 *        -shared -fPIC bcast_oracle.c -o libbcast_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

typedef long double real;

#define ORACLE_MAX_ARGS 24
#define ORACLE_MAX_OUT 4
#define ORACLE_MAX_DIMS 8

/* One scalar op: x[] are the N arguments (exact), xw the same arguments in the
 * working precision (float* or double*), y[] the M values, J[i*N + j] = dy_i/dx_j. */
typedef void (*scalar_fn)(int n, const real *x, const void *xw, int is_f64, real *y, real *J,
                          int *branch);

typedef struct {
  const char *name;
  int n_args; /* 0: any (variadic family) */
  int n_out;
  uint32_t nondiff_mask; /* bit j set: argument j is a control input, no partial */
  scalar_fn fn;
} op_desc;

static real sigm(real x) { return 1.0L / (1.0L + expl(-x)); }

/* ---- tanh(x*y + b)  ------------------------------------------------------- */
static void op_tanh_xy_b(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  real u = x[0] * x[1] + x[2];
  real t = tanhl(u);
  real d = 1.0L - t * t;
  y[0] = t;
  J[0] = d * x[1];
  J[1] = d * x[0];
  J[2] = d;
  *br = 0;
}

/* ---- HM-LSTM cell update with hidden state and biases -----------------------
 * Cell rule: the case equation of Sec. 3.1 (fused form in Sec. 3.2.3), with the
 * branch conditions read as: FLUSH if z == 1; COPY if z == 0 and z_below == 0;
 * UPDATE otherwise.  h' = sigma(o) tanh(c') except on COPY where h' = h.
 * Biases are added to the matching pre-activation.
 * args: f i o g c h z z_below b_f b_i b_o b_g ; outputs: c' h'
 * branch id: 0 UPDATE, 1 COPY, 2 FLUSH */
enum { A_F, A_I, A_O, A_G, A_C, A_H, A_Z, A_ZB, A_BF, A_BI, A_BO, A_BG, HM_N };
static void op_hmlstm(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64; /* z compares are exact in every precision */
  const int N = HM_N;
  real *Jc = J, *Jh = J + N;
  for (int k = 0; k < 2 * N; ++k) J[k] = 0.0L;
  real z = x[A_Z], zb = x[A_ZB];
  int flush = (z == 1.0L);
  if (!flush && z == 0.0L && zb == 0.0L) {
    y[0] = x[A_C];
    y[1] = x[A_H];
    Jc[A_C] = 1.0L;
    Jh[A_H] = 1.0L;
    *br = 1;
    return;
  }
  real si = sigm(x[A_I] + x[A_BI]);
  real tg = tanhl(x[A_G] + x[A_BG]);
  real so = sigm(x[A_O] + x[A_BO]);
  real cn = si * tg;
  Jc[A_I] = si * (1.0L - si) * tg;
  Jc[A_G] = si * (1.0L - tg * tg);
  if (!flush) {
    real sf = sigm(x[A_F] + x[A_BF]);
    cn += sf * x[A_C];
    Jc[A_F] = sf * (1.0L - sf) * x[A_C];
    Jc[A_C] = sf;
  }
  Jc[A_BF] = Jc[A_F];
  Jc[A_BI] = Jc[A_I];
  Jc[A_BG] = Jc[A_G];
  real tau = tanhl(cn);
  y[0] = cn;
  y[1] = so * tau;
  real dh_dc = so * (1.0L - tau * tau);
  Jh[A_F] = dh_dc * Jc[A_F];
  Jh[A_I] = dh_dc * Jc[A_I];
  Jh[A_G] = dh_dc * Jc[A_G];
  Jh[A_C] = dh_dc * Jc[A_C];
  Jh[A_O] = so * (1.0L - so) * tau;
  Jh[A_BF] = Jh[A_F];
  Jh[A_BI] = Jh[A_I];
  Jh[A_BG] = Jh[A_G];
  Jh[A_BO] = Jh[A_O];
  *br = flush ? 2 : 0;
}

/* ---- the paper's own fused cell update (Sec. 3.2.3), cell state only --------
 * args: c f i g z1 z2 ; z1 is the layer's previous boundary state, z2 the lower
 * layer's current one.  Same reading of the (overlapping) printed conditions. */
static void op_update_c(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  for (int k = 0; k < 6; ++k) J[k] = 0.0L;
  real c = x[0], z1 = x[4], z2 = x[5];
  if (z1 == 1.0L) {
    real si = sigm(x[2]), tg = tanhl(x[3]);
    y[0] = si * tg;
    J[2] = si * (1.0L - si) * tg;
    J[3] = si * (1.0L - tg * tg);
    *br = 2;
  } else if (z1 == 0.0L && z2 == 0.0L) {
    y[0] = c;
    J[0] = 1.0L;
    *br = 1;
  } else {
    real sf = sigm(x[1]), si = sigm(x[2]), tg = tanhl(x[3]);
    y[0] = sf * c + si * tg;
    J[0] = sf;
    J[1] = sf * (1.0L - sf) * c;
    J[2] = si * (1.0L - si) * tg;
    J[3] = si * (1.0L - tg * tg);
    *br = 0;
  }
}

/* ---- five-argument branchy broadcast ----------------------------------------
 * out = exp(-A) B + r  if A + s > t (sum rounded in the working precision)
 *     = log1p(A^2) r - s otherwise.   branch id: 1 = predicate true. */
static void op_branchy5(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n;
  int take;
  if (f64) {
    const double *w = (const double *)xw;
    volatile double sum = w[0] + w[3];
    take = sum > w[4];
  } else {
    const float *w = (const float *)xw;
    volatile float sum = w[0] + w[3];
    take = sum > w[4];
  }
  real A = x[0], B = x[1], r = x[2], s = x[3];
  if (take) {
    real e = expl(-A);
    y[0] = e * B + r;
    J[0] = -e * B;
    J[1] = e;
    J[2] = 1.0L;
    J[3] = 0.0L;
    J[4] = 0.0L;
  } else {
    real l = log1pl(A * A);
    y[0] = l * r - s;
    J[0] = 2.0L * A * r / (1.0L + A * A);
    J[1] = 0.0L;
    J[2] = l;
    J[3] = -1.0L;
    J[4] = 0.0L;
  }
  *br = take;
}

/* ---- small coverage ops -------------------------------------------------------*/
/* the paper's Dual example (Sec. 2.2.1): cos(Dual(x,y)) -> Dual(cos x, -sin x * y) */
static void op_cos_x(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  y[0] = cosl(x[0]);
  J[0] = -sinl(x[0]);
  *br = 0;
}
/* the elementary functions the other ops are built from, with their derivatives.  The
 * derivatives of sigma and tanh are written so that they keep their relative accuracy where the
 * functions saturate: sigma' = e / (1 + e)^2 with e = exp(-|x|), 1 - tanh^2 = 4 q / (1 + q)^2
 * with q = exp(-2 |x|) (identities; s (1 - s) and 1 - t^2 cancel there). */
static void op_elementary4(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  real e = expl(-fabsl(x[0])), q = expl(-2.0L * fabsl(x[0]));
  y[0] = expl(x[0]);
  J[0] = y[0];
  y[1] = log1pl(x[0]);
  J[1] = 1.0L / (1.0L + x[0]);
  y[2] = x[0] >= 0.0L ? 1.0L / (1.0L + e) : e / (1.0L + e);
  J[2] = e / ((1.0L + e) * (1.0L + e));
  y[3] = tanhl(x[0]);
  J[3] = 4.0L * q / ((1.0L + q) * (1.0L + q));
  *br = 0;
}
/* y = x * t : a scalar argument whose partial is not zero */
static void op_scale_xt(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  y[0] = x[0] * x[1];
  J[0] = x[1];
  J[1] = x[0];
  *br = 0;
}
/* b : R^3 -> R^2 (shape of the D(b) expansion in Sec. 2.2.2):
 * y1 = x1 x2 + sin x3 ; y2 = x1 / x2 - x3^2 */
static void op_pair3(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  y[0] = x[0] * x[1] + sinl(x[2]);
  y[1] = x[0] / x[1] - x[2] * x[2];
  J[0] = x[1];
  J[1] = x[0];
  J[2] = cosl(x[2]);
  J[3] = 1.0L / x[1];
  J[4] = -x[0] / (x[1] * x[1]);
  J[5] = -2.0L * x[2];
  *br = 0;
}
/* the HM-LSTM argument list with trivial arithmetic (a profiling aid of the library) */
static void op_linear12(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  (void)n; (void)xw; (void)f64;
  for (int k = 0; k < 24; ++k) J[k] = 0.0L;
  y[0] = x[A_Z] * x[A_ZB];
  for (int k = 0; k < HM_N; ++k)
    if (k != A_Z && k != A_ZB) { y[0] += x[k]; J[k] = 1.0L; }
  y[1] = x[A_F] * x[A_C] + x[A_I] * x[A_H] + x[A_O] * x[A_G] + x[A_BF] * x[A_BI] + x[A_BO] * x[A_BG];
  real *Jh = J + HM_N;
  Jh[A_F] = x[A_C]; Jh[A_C] = x[A_F]; Jh[A_I] = x[A_H]; Jh[A_H] = x[A_I]; Jh[A_O] = x[A_G]; Jh[A_G] = x[A_O];
  Jh[A_BF] = x[A_BI]; Jh[A_BI] = x[A_BF]; Jh[A_BO] = x[A_BG]; Jh[A_BG] = x[A_BO];
  *br = 0;
}

/* arity study (Sec. 3.4.1): f = prod_i tanh(g(x_i)), g(x) = x if x > 1/2 else -x.
 * branch id = number of arguments with x_i > 1/2. */
static void op_prod_tanh(int n, const real *x, const void *xw, int f64, real *y, real *J, int *br) {
  real t[ORACLE_MAX_ARGS], sg[ORACLE_MAX_ARGS];
  int cnt = 0;
  for (int k = 0; k < n; ++k) {
    int up = f64 ? (((const double *)xw)[k] > 0.5) : (((const float *)xw)[k] > 0.5f);
    cnt += up;
    sg[k] = up ? 1.0L : -1.0L;
    t[k] = tanhl(sg[k] * x[k]);
  }
  real p = 1.0L;
  for (int k = 0; k < n; ++k) p *= t[k];
  y[0] = p;
  for (int k = 0; k < n; ++k) {
    real others = 1.0L;
    for (int m = 0; m < n; ++m)
      if (m != k) others *= t[m];
    J[k] = others * (1.0L - t[k] * t[k]) * sg[k];
  }
  *br = cnt;
}

static const op_desc OPS[] = {
    {"hmlstm_update", HM_N, 2, (1u << A_Z) | (1u << A_ZB), op_hmlstm},
    {"tanh_xy_b", 3, 1, 0u, op_tanh_xy_b},
    {"branchy5", 5, 1, 0u, op_branchy5},
    {"update_c", 6, 1, (1u << 4) | (1u << 5), op_update_c},
    {"cos_x", 1, 1, 0u, op_cos_x},
    {"elementary4", 1, 4, 0u, op_elementary4},
    {"scale_xt", 2, 1, 0u, op_scale_xt},
    {"pair3", 3, 2, 0u, op_pair3},
    {"linear12", HM_N, 2, (1u << A_Z) | (1u << A_ZB), op_linear12},
    {"prod_tanh", 0, 1, 0u, op_prod_tanh},
};

static const op_desc *find_op(const char *name) {
  for (size_t k = 0; k < sizeof(OPS) / sizeof(OPS[0]); ++k)
    if (strcmp(OPS[k].name, name) == 0) return &OPS[k];
  return 0;
}

/* n_args/n_out/nondiff mask of an op; returns 0, or -1 for an unknown name. */
int oracle_op_info(const char *name, int *n_args, int *n_out, uint32_t *nondiff_mask) {
  const op_desc *op = find_op(name);
  if (!op) return -1;
  *n_args = op->n_args;
  *n_out = op->n_out;
  *nondiff_mask = op->nondiff_mask;
  return 0;
}

static real load(const void *p, int64_t off, int f64) {
  return f64 ? (real)((const double *)p)[off] : (real)((const float *)p)[off];
}
static void store(void *p, int64_t off, int f64, real v) {
  if (f64)
    ((double *)p)[off] = (double)v;
  else
    ((float *)p)[off] = (float)v;
}

/* offset of output multi-index idx[] inside a contiguous row-major array of the
 * given shape, size-1 dims indexed at 0 */
static int64_t bcast_offset(int ndim, const int64_t *idx, const int64_t *shape) {
  int64_t off = 0;
  for (int d = 0; d < ndim; ++d) off = off * shape[d] + (shape[d] == 1 ? 0 : idx[d]);
  return off;
}

/*
 * Forward.  All arrays are contiguous row-major at full rank `ndim`;
 * arg_shapes[j*ndim + d] is either out_shape[d] or 1.  outs: M arrays of the
 * output shape; partials: M * N_d arrays of the output shape in the order
 * [i * N_d + jd] where jd counts differentiable arguments in argument order;
 * branch: optional E bytes.  Returns 0, -1 unknown op, -2 bad argument count,
 * -3 shape error.
 */
int oracle_forward(const char *name, int is_f64, int ndim, const int64_t *out_shape, int n_args,
                   const void *const *args, const int64_t *arg_shapes, void *const *outs,
                   void *const *partials, uint8_t *branch, int n_threads) {
  const op_desc *op = find_op(name);
  if (!op) return -1;
  if ((op->n_args && op->n_args != n_args) || n_args < 1 || n_args > ORACLE_MAX_ARGS) return -2;
  if (ndim < 1 || ndim > ORACLE_MAX_DIMS) return -3;
  int64_t E = 1;
  for (int d = 0; d < ndim; ++d) E *= out_shape[d];
  for (int j = 0; j < n_args; ++j)
    for (int d = 0; d < ndim; ++d) {
      int64_t s = arg_shapes[j * ndim + d];
      if (s != out_shape[d] && s != 1) return -3;
    }
  const int N = n_args, M = op->n_out;
  int jd_of[ORACLE_MAX_ARGS], Nd = 0;
  for (int j = 0; j < N; ++j) jd_of[j] = ((op->nondiff_mask >> j) & 1u) ? -1 : Nd++;
  if (n_threads < 1) n_threads = 1;

#pragma omp parallel for num_threads(n_threads) schedule(static)
  for (int64_t e = 0; e < E; ++e) {
    int64_t idx[ORACLE_MAX_DIMS];
    int64_t rem = e;
    for (int d = ndim - 1; d >= 0; --d) {
      idx[d] = rem % out_shape[d];
      rem /= out_shape[d];
    }
    real x[ORACLE_MAX_ARGS];
    double xd[ORACLE_MAX_ARGS];
    float xf[ORACLE_MAX_ARGS];
    for (int j = 0; j < N; ++j) {
      int64_t off = bcast_offset(ndim, idx, arg_shapes + j * ndim);
      x[j] = load(args[j], off, is_f64);
      xd[j] = (double)x[j];
      xf[j] = (float)x[j];
    }
    real y[ORACLE_MAX_OUT], J[ORACLE_MAX_OUT * ORACLE_MAX_ARGS];
    int br = 0;
    op->fn(N, x, is_f64 ? (const void *)xd : (const void *)xf, is_f64, y, J, &br);
    for (int i = 0; i < M; ++i) {
      store(outs[i], e, is_f64, y[i]);
      for (int j = 0; j < N; ++j)
        if (jd_of[j] >= 0 && partials) store(partials[i * Nd + jd_of[j]], e, is_f64, J[i * N + j]);
    }
    if (branch) branch[e] = (uint8_t)br;
  }
  return 0;
}

/* Neumaier-compensated accumulation in long double.  The compensation term estimates the
 * rounding error of finite additions; once a term or the running sum is infinite or NaN it is
 * itself inf - inf, so the result is then the plain IEEE sum (an infinity among finite terms
 * stays that infinity, as Table 1's sum of products says it must). */
typedef struct { real s, c; } csum;
static real csum_value(const csum *a) { return isfinite(a->s) ? a->s + a->c : a->s; }
static void csum_add(csum *a, real v) {
  real t = a->s + v;
  if (fabsl(a->s) >= fabsl(v))
    a->c += (a->s - t) + v;
  else
    a->c += (v - t) + a->s;
  a->s = t;
}

/*
 * Backward (op independent).  adjoints: M arrays of the output shape; partials:
 * the M * N_d arrays in forward's order; grad_shapes[jd*ndim + d] is out_shape[d]
 * or 1; grads: N_d arrays of those shapes.  Every array contiguous row-major.
 * A NULL partial plane stands for a plane of zeros.
 */
int oracle_backward(int is_f64, int ndim, const int64_t *out_shape, int M, int Nd,
                    const void *const *adjoints, const void *const *partials,
                    const int64_t *grad_shapes, void *const *grads, int n_threads) {
  if (ndim < 1 || ndim > ORACLE_MAX_DIMS || M < 1 || M > ORACLE_MAX_OUT || Nd < 1) return -3;
  for (int j = 0; j < Nd; ++j)
    for (int d = 0; d < ndim; ++d) {
      int64_t s = grad_shapes[j * ndim + d];
      if (s != out_shape[d] && s != 1) return -3;
    }
  if (n_threads < 1) n_threads = 1;
  for (int j = 0; j < Nd; ++j) {
    const int64_t *gs = grad_shapes + j * ndim;
    int64_t G = 1, F = 1; /* gradient elements; elements each one was expanded to */
    int64_t fshape[ORACLE_MAX_DIMS];
    for (int d = 0; d < ndim; ++d) {
      G *= gs[d];
      fshape[d] = (gs[d] == 1) ? out_shape[d] : 1;
      F *= fshape[d];
    }
#pragma omp parallel for num_threads(n_threads) schedule(static)
    for (int64_t a = 0; a < G; ++a) {
      int64_t aidx[ORACLE_MAX_DIMS], idx[ORACLE_MAX_DIMS];
      int64_t rem = a;
      for (int d = ndim - 1; d >= 0; --d) {
        aidx[d] = rem % gs[d];
        rem /= gs[d];
      }
      csum acc = {0.0L, 0.0L};
      for (int64_t q = 0; q < F; ++q) {
        int64_t qr = q;
        for (int d = ndim - 1; d >= 0; --d) {
          int64_t k = qr % fshape[d];
          qr /= fshape[d];
          idx[d] = (gs[d] == 1) ? k : aidx[d];
        }
        int64_t e = bcast_offset(ndim, idx, out_shape);
        for (int i = 0; i < M; ++i) {
          const void *P = partials[i * Nd + j];
          /* an absent plane is a plane of zeros: its products are adjoint x 0 (NaN for a non-finite adjoint) */
          csum_add(&acc, load(adjoints[i], e, is_f64) * (P ? load(P, e, is_f64) : 0.0L));
        }
      }
      store(grads[j], a, is_f64, csum_value(&acc));
    }
  }
  return 0;
}
