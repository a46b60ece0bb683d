// Built-in op table: each entry is ONE scalar function b : R^N -> R^M, already the fused
// composition of its broadcasts (Sec. 2.1.2), written once over a generic number type.
// The forward kernel instantiates it on dual numbers seeded x_j + eps_j (the D operator,
// Sec. 2.2.2), so the data-dependent `if`s below run per element inside the kernel and
// only the taken branch is differentiated (Sec. 2.2.4, point 3).
//
// Contract of an op:  static int apply(Y *y, const X&... x)
//   x...  the N arguments in op order; differentiable ones are duals, control inputs
//         (bits of NONDIFF) are plain scalars
//   y[M]  outputs, duals over all N_d perturbations (narrower results widen on assignment)
//   returns the branch id taken (0 .. NBR-1)
// STRIDED: the tiled forward kernel is also built for views whose row strides differ from one
// another (arguments that are slices of wider buffers); ops without it take the generic strided
// kernels in that case.
// RECOMPUTE_PATTERN names the broadcast pattern the recompute-in-reverse kernel is also compiled
// for without run-time dispatch: 3 bits per differentiable argument, 1 = full shape, 2 = varies
// along rows only (gradient = row sums), 3 = varies along columns only (column sums), 4 = scalar.
#pragma once
#include "dual.h"

namespace bd {

// out = tanh(x*y + b)
struct OpTanhXyB {
  static constexpr int N = 3, M = 1, NBR = 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x89ull;
  template <class Y, class X0, class X1, class B>
  static BD_DEV int apply(Y *y, const X0 &x, const X1 &w, const B &b) {
    y[0] = tanh(x * w + b);
    return 0;
  }
};

// HM-LSTM cell update (Sec. 3.1 case equation; fused scalar form of Sec. 3.2.3) extended
// with the hidden state, the output gate and per-gate biases.
// args: f i o g c h z z_below b_f b_i b_o b_g  ->  (c', h').  FLUSH if z == 1; COPY if
// z == 0 and z_below == 0; UPDATE otherwise (so off-grid control values fall to UPDATE).
// FLUSH and UPDATE share the sigma(i) tanh(g) term, written once so that a wavefront
// holding both branches evaluates it once.
struct OpHmLstmUpdate {
  static constexpr int N = 12, M = 2, NBR = 3;
  static constexpr uint32_t NONDIFF = (1u << 6) | (1u << 7);
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x12489249ull;
  template <class Y, class F, class I, class O, class G, class C, class H, class Z, class BF, class BI,
            class BO, class BG>
  static BD_DEV int apply(Y *y, const F &f, const I &i, const O &o, const G &g, const C &c, const H &h,
                          const Z &z, const Z &zb, const BF &bf, const BI &bi, const BO &bo, const BG &bg) {
    using T = typename Y::value_type;
    const bool flush = (z == T(1));
    if (!flush && z == T(0) && zb == T(0)) {  // COPY
      y[0] = c;
      y[1] = h;
      return 1;
    }
    using CN = decltype(sigmoid(f + bf) * c + sigmoid(i + bi) * tanh(g + bg));
    CN cn = sigmoid(i + bi) * tanh(g + bg);
    if (!flush) cn = cn + sigmoid(f + bf) * c;  // UPDATE keeps the old cell through the forget gate
    y[0] = cn;
    y[1] = sigmoid(o + bo) * tanh(cn);
    return flush ? 2 : 0;
  }
};

// The paper's six-argument fused update (Sec. 3.2.3): args c f i g z1 z2 -> c'.
struct OpUpdateC {
  static constexpr int N = 6, M = 1, NBR = 3;
  static constexpr uint32_t NONDIFF = (1u << 4) | (1u << 5);
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x249ull;
  template <class Y, class C, class F, class I, class G, class Z>
  static BD_DEV int apply(Y *y, const C &c, const F &f, const I &i, const G &g, const Z &z1, const Z &z2) {
    using T = typename Y::value_type;
    if (z1 == T(1)) {  // FLUSH
      y[0] = sigmoid(i) * tanh(g);
      return 2;
    } else if (z1 == T(0) && z2 == T(0)) {  // COPY
      y[0] = c;
      return 1;
    }
    y[0] = sigmoid(f) * c + sigmoid(i) * tanh(g);  // UPDATE
    return 0;
  }
};

// out = exp(-A)*B + r  if A + s > t  else  log1p(A*A)*r - s.   The predicate is evaluated
// exactly as written, in the working precision.
struct OpBranchy5 {
  static constexpr int N = 5, M = 1, NBR = 2;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x44c9ull;
  template <class Y, class A, class B, class R, class S, class TT>
  static BD_DEV int apply(Y *y, const A &a, const B &b, const R &r, const S &s, const TT &t) {
    if (a + s > t) {
      y[0] = exp(-a) * b + r;
      return 1;
    }
    y[0] = log1p(a * a) * r - s;
    return 0;
  }
};

// (exp x, log1p x, sigma x, tanh x): the elementary functions the other ops are built from, each
// with its derivative -- exposed so that their accuracy can be measured over their whole domain
struct OpElementary4 {
  static constexpr int N = 1, M = 4, NBR = 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x1ull;
  template <class Y, class X>
  static BD_DEV int apply(Y *y, const X &x) {
    y[0] = exp(x);
    y[1] = log1p(x);
    y[2] = sigmoid(x);
    y[3] = tanh(x);
    return 0;
  }
};

// cos(x): the Dual example of Sec. 2.2.1
struct OpCosX {
  static constexpr int N = 1, M = 1, NBR = 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x1ull;
  template <class Y, class X>
  static BD_DEV int apply(Y *y, const X &x) {
    y[0] = cos(x);
    return 0;
  }
};

// x * t
struct OpScaleXt {
  static constexpr int N = 2, M = 1, NBR = 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x21ull;
  template <class Y, class X, class TT>
  static BD_DEV int apply(Y *y, const X &x, const TT &t) {
    y[0] = x * t;
    return 0;
  }
};

// b : R^3 -> R^2, (x1*x2 + sin x3, x1/x2 - x3*x3)
struct OpPair3 {
  static constexpr int N = 3, M = 2, NBR = 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0xa1ull;
  template <class Y, class X1, class X2, class X3>
  static BD_DEV int apply(Y *y, const X1 &x1, const X2 &x2, const X3 &x3) {
    y[0] = x1 * x2 + sin(x3);
    y[1] = x1 / x2 - x3 * x3;
    return 0;
  }
};

// An arithmetic-light op with the argument list of the HM-LSTM update (same planes, same
// traffic, almost no math): separates memory behaviour from arithmetic when profiling.
struct OpLinear12 {
  static constexpr int N = 12, M = 2, NBR = 1;
  static constexpr uint32_t NONDIFF = (1u << 6) | (1u << 7);
  static constexpr bool STRIDED = true;
  static constexpr uint64_t RECOMPUTE_PATTERN = 0x12489249ull;
  template <class Y, class F, class I, class O, class G, class C, class H, class Z, class BF, class BI,
            class BO, class BG>
  static BD_DEV int apply(Y *y, const F &f, const I &i, const O &o, const G &g, const C &c, const H &h,
                          const Z &z, const Z &zb, const BF &bf, const BI &bi, const BO &bo, const BG &bg) {
    y[0] = f + i + o + g + c + h + bf + bi + bo + bg + z * zb;
    y[1] = f * c + i * h + o * g + bf * bi + bo * bg;
    return 0;
  }
};

// Arity study (Sec. 3.4.1): prod_i tanh(g(x_i)), g(x) = x if x > 1/2 else -x.
template <int ARITY>
struct OpProdTanh {
  static constexpr int N = ARITY, M = 1, NBR = ARITY + 1;
  static constexpr uint32_t NONDIFF = 0u;
  static constexpr bool STRIDED = false;
  static constexpr uint64_t all_full() {
    uint64_t q = 0;
    for (int j = 0; j < ARITY; ++j) q |= 1ull << (3 * j);
    return q;
  }
  static constexpr uint64_t RECOMPUTE_PATTERN = all_full();
  template <class X>
  static BD_DEV X g(const X &x) {
    using T = typename X::value_type;
    if (x > T(0.5)) return x;
    return -x;
  }
  template <class Y, class... X>
  static BD_DEV int apply(Y *y, const X &...x) {
    using T = typename Y::value_type;
    y[0] = (tanh(g(x)) * ...);
    return (0 + ... + int(x > T(0.5)));
  }
};

}  // namespace bd
