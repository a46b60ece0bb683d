// Multidimensional dual numbers for device code (Sec. 2.2.1 of arXiv 1810.08297).
//
// x + sum_k y_k eps_k with eps_i eps_j = 0.  A Dual carries its value and one partial
// per perturbation it can depend on.  WHICH perturbations those are is part of the
// type (MASK, one bit per differentiable argument of the broadcast): the sum of two
// duals has the union of their masks, a seed has one bit.  Partials that are
// structurally zero therefore never occupy a register and are never multiplied --
// the dead-partial elimination does not depend on floating-point folding rules.
// Comparisons read the value part only, so control flow adds no derivative.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

namespace bd {

#define BD_DEV __device__ __forceinline__

constexpr int BD_MAX_BITS = 20;

constexpr int popc(uint32_t m) { return __builtin_popcount(m); }
constexpr int slot_of(uint32_t mask, int bit) { return popc(mask & ((1u << bit) - 1u)); }

template <int I, int N, class F>
BD_DEV void static_for(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// ---- scalar math in the working precision ------------------------------------------
template <class T> struct smath;
template <> struct smath<float> {
  // 2^(x log2 e): the rounding error of the product and of the float constant is folded
  // back in as 2^t (1 + err ln 2); v_exp_f32 is accurate to 1 ulp.  About 1.5 ulp overall.
  // Where 2^t is not finite (it overflows from t = 128 on, the residual can have either sign
  // there and inf * err + inf would be NaN for a negative one) or the argument is infinite
  // (the residual is inf - inf) the correction is left out: underflow gives 0, overflow and
  // +inf give inf, -inf gives 0.
  static BD_DEV float exp(float x) {
    const float L2E = 1.44269504088896340736f;
    float t = x * L2E;
    float e = ::fmaf(x, L2E, -t);
    e = ::fmaf(x, 1.925963033500e-8f, e);
    float p = __builtin_amdgcn_exp2f(t);
    return (::fabsf(t) < 160.0f && __builtin_isfinite(p)) ? ::fmaf(p, e * 0.6931471805599453f, p) : p;
  }
  // log(u) + (x - (u - 1)) / u with u = fl(1 + x): the second term gives back what the
  // rounding of 1 + x dropped, so tiny x return x and nothing cancels.  log(u) is the hardware
  // log2 (1 ulp) times ln 2, the constant's own rounding error folded in.  About 2 ulp.
  static BD_DEV float log1p(float x) {
    const float u = 1.0f + x;
    const float l2 = __builtin_amdgcn_logf(u);
    float l = l2 * 0.693147182464599609375f;  // ln 2 rounded to float ...
    const float lr = ::fmaf(l2, -1.904654323148236e-9f, l);  // ... and the remainder of ln 2
    l = __builtin_isfinite(l2) ? lr : l;  // log2 of inf or of 0: the correction would be inf - inf
    const float lost = x - (u - 1.0f);
    return (x > 3.0e38f || u == 0.0f) ? l : ::fmaf(lost, __builtin_amdgcn_rcpf(u), l);  // inf and -1 pass through
  }
  static BD_DEV float sin(float x) { return ::sinf(x); }
  static BD_DEV float cos(float x) { return ::cosf(x); }
  static BD_DEV float abs(float x) { return ::fabsf(x); }
  static BD_DEV float copysign(float m, float s) { return ::copysignf(m, s); }
  // hardware reciprocal (1 ulp) refined by one Newton step; where the step has no finite result
  // (d = 0 or infinite: 0 * inf) the hardware's own inf or 0 stands
  static BD_DEV float rcp(float d) {
    const float r = __builtin_amdgcn_rcpf(d);
    const float n = ::fmaf(::fmaf(-d, r, 1.0f), r, r);
    return __builtin_isfinite(n) ? n : r;
  }
  // the same for 1 <= d <= 2 (or NaN), where the step always has its result
  static BD_DEV float rcp_1to2(float d) {
    const float r = __builtin_amdgcn_rcpf(d);
    return ::fmaf(::fmaf(-d, r, 1.0f), r, r);
  }
};
template <> struct smath<double> {
  static BD_DEV double exp(double x) { return ::exp(x); }
  static BD_DEV double log1p(double x) { return ::log1p(x); }
  static BD_DEV double sin(double x) { return ::sin(x); }
  static BD_DEV double cos(double x) { return ::cos(x); }
  static BD_DEV double abs(double x) { return ::fabs(x); }
  static BD_DEV double copysign(double m, double s) { return ::copysign(m, s); }
  static BD_DEV double rcp(double d) { return 1.0 / d; }
  static BD_DEV double rcp_1to2(double d) { return 1.0 / d; }
};

// sigma(x) and sigma'(x) from e = exp(-|x|): no overflow, no cancellation
template <class T>
BD_DEV void sigmoid_vd(T x, T &s, T &ds) {
  T e = smath<T>::exp(-smath<T>::abs(x));
  T r = smath<T>::rcp_1to2(T(1) + e);
  T er = e * r;
  s = x >= T(0) ? r : er;
  ds = er * r;
}
// tanh(x) and 1 - tanh^2(x) from q = exp(-2|x|): the derivative keeps full relative
// accuracy where tanh saturates.  tanh itself is (1 - q) / (1 + q), which cancels for small
// |x| (q -> 1): there the odd power series takes over, through x^11 below 0.35 in fp32 (remainder
// under a fifth of a unit in the last place) and through x^23 below 0.25 in fp64.
BD_DEV void tanh_vd(float x, float &t, float &dt) {
  const float a = smath<float>::abs(x);
  const float q = smath<float>::exp(-2.0f * a);
  const float r = smath<float>::rcp_1to2(1.0f + q);
  const float x2 = x * x;
  float s = ::fmaf(x2, -8.86323550e-3f, 2.18694885e-2f);  // -1382/155925, 62/2835
  s = ::fmaf(x2, s, -5.39682540e-2f);                     // -17/315
  s = ::fmaf(x2, s, 1.33333333e-1f);                      // 2/15
  s = ::fmaf(x2, s, -3.33333333e-1f);                     // -1/3
  s = ::fmaf(x * x2, s, x);
  t = a < 0.35f ? s : smath<float>::copysign((1.0f - q) * r, x);
  dt = 4.0f * q * r * r;
}
BD_DEV void tanh_vd(double x, double &t, double &dt) {
  const double a = smath<double>::abs(x);
  const double q = smath<double>::exp(-2.0 * a);
  const double r = smath<double>::rcp(1.0 + q);
  // 2^(2n) (2^(2n) - 1) B_2n / (2n)!, n = 12 .. 2: the series through x^23, remainder below 1e-19 for |x| < 0.25
  const double c[11] = {-3.927832388331683e-05, 9.691537956929451e-05, -0.00023912911424355248, 0.000590027440945586,
                        -0.0014558343870513183, 0.003592128036572481, -0.008863235529902197, 0.021869488536155203,
                        -0.05396825396825397, 0.13333333333333333, -0.3333333333333333};
  const double x2 = x * x;
  double s = c[0];
#pragma unroll
  for (int k = 1; k < 11; ++k) s = __builtin_fma(x2, s, c[k]);
  s = __builtin_fma(x * x2, s, x);
  t = a < 0.25 ? s : smath<double>::copysign((1.0 - q) * r, x);
  dt = 4.0 * q * r * r;
}

// ---- the dual type -------------------------------------------------------------------
template <class T, uint32_t MASK>
struct Dual {
  using value_type = T;
  static constexpr uint32_t mask = MASK;
  static constexpr int K = popc(MASK);
  T v;
  T d[K > 0 ? K : 1];

  BD_DEV Dual() {}
  BD_DEV explicit Dual(T value) : v(value) {
    for (int k = 0; k < (K > 0 ? K : 1); ++k) d[k] = T(0);
  }
  // widening: a dual that depends on fewer perturbations, zero elsewhere
  template <uint32_t SUB, class = std::enable_if_t<(SUB & ~MASK) == 0 && SUB != MASK>>
  BD_DEV Dual(const Dual<T, SUB> &o) : v(o.v) {
    static_for<0, BD_MAX_BITS>([&](auto B) {
      constexpr int bit = decltype(B)::value;
      if constexpr ((MASK >> bit) & 1u) d[slot_of(MASK, bit)] = o.template partial<bit>();
    });
  }
  // tangent extraction (the tg operator of Sec. 2.2.1) for one perturbation
  template <int BIT>
  BD_DEV T partial() const {
    if constexpr ((MASK >> BIT) & 1u)
      return d[slot_of(MASK, BIT)];
    else
      return T(0);
  }
};

template <class X> struct is_dual : std::false_type {};
template <class T, uint32_t M> struct is_dual<Dual<T, M>> : std::true_type {};

// seed x + eps_bit
template <class T, int BIT>
BD_DEV Dual<T, (1u << BIT)> seed(T x) {
  Dual<T, (1u << BIT)> r;
  r.v = x;
  r.d[0] = T(1);
  return r;
}

// r = value v with partials fa(a') + fb(b') over the union of the masks
template <class T, uint32_t MA, uint32_t MB, class FA, class FB>
BD_DEV Dual<T, (MA | MB)> zip(T v, const Dual<T, MA> &a, const Dual<T, MB> &b, FA fa, FB fb) {
  constexpr uint32_t MR = MA | MB;
  Dual<T, MR> r;
  r.v = v;
  static_for<0, BD_MAX_BITS>([&](auto B) {
    constexpr int bit = decltype(B)::value;
    if constexpr ((MR >> bit) & 1u) {
      constexpr bool ina = (MA >> bit) & 1u, inb = (MB >> bit) & 1u;
      if constexpr (ina && inb)
        r.d[slot_of(MR, bit)] = fa(a.template partial<bit>()) + fb(b.template partial<bit>());
      else if constexpr (ina)
        r.d[slot_of(MR, bit)] = fa(a.template partial<bit>());
      else
        r.d[slot_of(MR, bit)] = fb(b.template partial<bit>());
    }
  });
  return r;
}
// unary chain rule: f(x + y eps) = f(x) + f'(x) y eps
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> chain(T v, T dv, const Dual<T, MA> &a) {
  Dual<T, MA> r;
  r.v = v;
  for (int k = 0; k < Dual<T, MA>::K; ++k) r.d[k] = dv * a.d[k];
  return r;
}

// ---- arithmetic ---------------------------------------------------------------------
template <class T, uint32_t MA, uint32_t MB>
BD_DEV auto operator+(const Dual<T, MA> &a, const Dual<T, MB> &b) {
  return zip(a.v + b.v, a, b, [](T x) { return x; }, [](T x) { return x; });
}
template <class T, uint32_t MA, uint32_t MB>
BD_DEV auto operator-(const Dual<T, MA> &a, const Dual<T, MB> &b) {
  return zip(a.v - b.v, a, b, [](T x) { return x; }, [](T x) { return -x; });
}
template <class T, uint32_t MA, uint32_t MB>
BD_DEV auto operator*(const Dual<T, MA> &a, const Dual<T, MB> &b) {
  const T av = a.v, bv = b.v;
  return zip(av * bv, a, b, [bv](T x) { return x * bv; }, [av](T x) { return x * av; });
}
template <class T, uint32_t MA, uint32_t MB>
BD_DEV auto operator/(const Dual<T, MA> &a, const Dual<T, MB> &b) {
  const T inv = smath<T>::rcp(b.v);
  const T q = a.v * inv;
  const T mq = -q * inv;
  return zip(q, a, b, [inv](T x) { return x * inv; }, [mq](T x) { return x * mq; });
}
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator-(const Dual<T, MA> &a) { return chain(-a.v, T(-1), a); }

// dual (op) plain scalar
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator+(const Dual<T, MA> &a, T s) { Dual<T, MA> r = a; r.v = a.v + s; return r; }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator+(T s, const Dual<T, MA> &a) { return a + s; }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator-(const Dual<T, MA> &a, T s) { Dual<T, MA> r = a; r.v = a.v - s; return r; }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator-(T s, const Dual<T, MA> &a) { return chain(s - a.v, T(-1), a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator*(const Dual<T, MA> &a, T s) { return chain(a.v * s, s, a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> operator*(T s, const Dual<T, MA> &a) { return chain(a.v * s, s, a); }

// ---- comparisons: value part only -----------------------------------------------------
template <class X> BD_DEV auto val(const X &x) {
  if constexpr (is_dual<X>::value) return x.v; else return x;
}
#define BD_CMP(OP)                                                                              \
  template <class A, class B, class = std::enable_if_t<is_dual<A>::value || is_dual<B>::value>> \
  BD_DEV bool operator OP(const A &a, const B &b) { return val(a) OP val(b); }
BD_CMP(>)
BD_CMP(<)
BD_CMP(>=)
BD_CMP(<=)
BD_CMP(==)
BD_CMP(!=)
#undef BD_CMP

// ---- elementary functions -------------------------------------------------------------
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> exp(const Dual<T, MA> &a) { T e = smath<T>::exp(a.v); return chain(e, e, a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> log1p(const Dual<T, MA> &a) {
  return chain(smath<T>::log1p(a.v), smath<T>::rcp(T(1) + a.v), a);
}
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> sin(const Dual<T, MA> &a) { return chain(smath<T>::sin(a.v), smath<T>::cos(a.v), a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> cos(const Dual<T, MA> &a) { return chain(smath<T>::cos(a.v), -smath<T>::sin(a.v), a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> sigmoid(const Dual<T, MA> &a) { T s, ds; sigmoid_vd(a.v, s, ds); return chain(s, ds, a); }
template <class T, uint32_t MA>
BD_DEV Dual<T, MA> tanh(const Dual<T, MA> &a) { T t, dt; tanh_vd(a.v, t, dt); return chain(t, dt, a); }

}  // namespace bd
