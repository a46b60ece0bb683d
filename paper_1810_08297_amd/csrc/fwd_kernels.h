// Dual-number forward kernels: one launch evaluates b on x_j + eps_j for every element and
// writes the M values and the M x N_d partial planes (Sec. 2.2.2; fused primal + tangent
// evaluation, Sec. 2.2.3).  HBM-bound: no matrix cores; the work is laid out so that every
// wavefront memory instruction moves 64 x 16 contiguous bytes per plane.
#pragma once
#include <hip/hip_runtime.h>

#include "kparams.h"
#include "ops.h"

namespace bd {

template <class T, int VEC> struct vec_of;
template <> struct vec_of<float, 4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct vec_of<double, 2> { typedef double type __attribute__((ext_vector_type(2))); };

template <class T, int VEC>
BD_DEV void load_vec(const T *p, T (&x)[VEC]) {
  if constexpr (VEC == 1) {
    x[0] = *p;
  } else {
    using V = typename vec_of<T, VEC>::type;
    V v = *reinterpret_cast<const V *>(p);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = v[k];
  }
}
template <class T, int VEC>
BD_DEV void store_vec(T *p, const T (&x)[VEC], bool nt) {
  if constexpr (VEC == 1) {
    if (nt) __builtin_nontemporal_store(x[0], p); else *p = x[0];
  } else {
    using V = typename vec_of<T, VEC>::type;
    V v;
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = x[k];
    if (nt) __builtin_nontemporal_store(v, reinterpret_cast<V *>(p)); else *reinterpret_cast<V *>(p) = v;
  }
}

// one argument for VEC consecutive columns of row r: a vector load where the argument
// varies along the columns, one element replicated where it is stride-0 there
template <class T, int VEC>
BD_DEV void load_arg(const TView &a, int64_t r, int64_t c0, T (&x)[VEC]) {
  const T *base = static_cast<const T *>(a.p) + r * a.sr;
  if (a.sc != 0) {
    load_vec<T, VEC>(base + c0, x);
  } else {
    T s = *base;
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = s;
  }
}

template <class Op, class T, int J>
BD_DEV auto make_arg(T x) {
  if constexpr ((Op::NONDIFF >> J) & 1u)
    return x;  // control input: a plain scalar, no perturbation
  else
    return seed<T, popc(~Op::NONDIFF & ((1u << J) - 1u))>(x);
}
template <class Op, class T, int VEC, class Y, size_t... J>
BD_DEV int eval_op(const T (&a)[Op::N][VEC], int v, Y *y, std::index_sequence<J...>) {
  return Op::apply(y, make_arg<Op, T, (int)J>(a[J][v])...);
}

// Tiled 2-D kernel.  Block = 256 lanes arranged TY x TX; a lane owns VEC consecutive
// columns and walks `steps` rows spaced TY apart.  Arguments that do not vary along the
// rows (row vectors, scalars) are loaded once and stay in registers for the whole walk;
// arguments that do not vary along the columns are one broadcast load per row.
template <class Op, class T, int VEC>
__global__ __launch_bounds__(kBlock) void fwd_tiled_kernel(const FwdTiledParams p) {
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  const int ltx = p.log2_tx;
  const int tx = threadIdx.x & ((1 << ltx) - 1);
  const int ty = threadIdx.x >> ltx;
  const int TY = kBlock >> ltx;
  const uint32_t nct = (uint32_t)p.n_ct;
  const uint32_t rt = blockIdx.x / nct, ct = blockIdx.x - rt * nct;
  const int64_t c0 = ((((int64_t)ct) << ltx) + tx) * VEC;
  if (c0 >= p.C) return;
  int64_t r = (int64_t)rt * ((int64_t)TY * p.steps) + ty;
  const bool nt = p.nt_store != 0;

  T a[N][VEC];
#pragma unroll
  for (int j = 0; j < N; ++j)
    if (p.arg[j].sr == 0) load_arg<T, VEC>(p.arg[j], 0, c0, a[j]);

  for (int k = 0; k < p.steps && r < p.R; ++k, r += TY) {
#pragma unroll
    for (int j = 0; j < N; ++j)
      if (p.arg[j].sr != 0) load_arg<T, VEC>(p.arg[j], r, c0, a[j]);

    Y y[VEC][M];
    int br[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) br[v] = eval_op<Op, T, VEC>(a, v, y[v], std::make_index_sequence<N>{});

    T o[VEC];
#pragma unroll
    for (int i = 0; i < M; ++i) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) o[v] = y[v][i].v;
      store_vec<T, VEC>(static_cast<T *>(p.out[i].p) + r * p.out[i].sr + c0, o, nt);
    }
    if (p.has_partials) {
#pragma unroll
      for (int i = 0; i < M; ++i) {
        static_for<0, ND>([&](auto JD) {
          constexpr int jd = decltype(JD)::value;
          const TView &pl = p.part[i * ND + jd];
          if (pl.p != nullptr) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) o[v] = y[v][i].template partial<jd>();
            store_vec<T, VEC>(static_cast<T *>(pl.p) + r * pl.sr + c0, o, nt);
          }
        });
      }
    }
    if (p.branch.p != nullptr) {
      uint8_t *bp = static_cast<uint8_t *>(p.branch.p) + r * p.branch.sr + c0 * p.branch.sc;
      if (VEC == 4 && p.branch.sc == 1 && (reinterpret_cast<uintptr_t>(bp) & 3u) == 0) {
        uint32_t w = 0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) w |= (uint32_t)(br[v] & 0xff) << (8 * v);
        *reinterpret_cast<uint32_t *>(bp) = w;
      } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) bp[v * p.branch.sc] = (uint8_t)br[v];
      }
    }
  }
}

// Generic kernel: any rank up to BCAST_MAX_DIMS, any strides; one element per lane.
template <class Op, class T>
__global__ __launch_bounds__(kBlock) void fwd_generic_kernel(const FwdGenericParams p) {
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= p.E) return;
  int64_t idx[BCAST_MAX_DIMS] = {0, 0, 0, 0};
  {
    int64_t rem = e;
#pragma unroll
    for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
      if (d < p.nd) {
        idx[d] = rem % p.shape[d];
        rem /= p.shape[d];
      }
  }
  auto off = [&](const GView &g) {
    int64_t o = 0;
#pragma unroll
    for (int d = 0; d < BCAST_MAX_DIMS; ++d) o += idx[d] * g.s[d];
    return o;
  };
  T a[N][1];
#pragma unroll
  for (int j = 0; j < N; ++j) a[j][0] = static_cast<const T *>(p.arg[j].p)[off(p.arg[j])];
  Y y[M];
  const int br = eval_op<Op, T, 1>(a, 0, y, std::make_index_sequence<N>{});
#pragma unroll
  for (int i = 0; i < M; ++i) {
    static_cast<T *>(p.out[i].p)[off(p.out[i])] = y[i].v;
    static_for<0, ND>([&](auto JD) {
      constexpr int jd = decltype(JD)::value;
      const GView &pl = p.part[i * ND + jd];
      if (pl.p != nullptr) static_cast<T *>(pl.p)[off(pl)] = y[i].template partial<jd>();
    });
  }
  if (p.branch.p != nullptr) static_cast<uint8_t *>(p.branch.p)[off(p.branch)] = (uint8_t)br;
}

// ---- launch wrappers, one pair per op ------------------------------------------------------
template <class Op>
hipError_t launch_fwd_tiled(int dt, int vec, const FwdTiledParams &p, dim3 grid, hipStream_t s) {
  if (dt == BCAST_F32) {
    if (vec > 1)
      hipLaunchKernelGGL((fwd_tiled_kernel<Op, float, 4>), grid, dim3(kBlock), 0, s, p);
    else
      hipLaunchKernelGGL((fwd_tiled_kernel<Op, float, 1>), grid, dim3(kBlock), 0, s, p);
  } else {
    if (vec > 1)
      hipLaunchKernelGGL((fwd_tiled_kernel<Op, double, 2>), grid, dim3(kBlock), 0, s, p);
    else
      hipLaunchKernelGGL((fwd_tiled_kernel<Op, double, 1>), grid, dim3(kBlock), 0, s, p);
  }
  return hipGetLastError();
}
template <class Op>
hipError_t launch_fwd_generic(int dt, const FwdGenericParams &p, dim3 grid, hipStream_t s) {
  if (dt == BCAST_F32)
    hipLaunchKernelGGL((fwd_generic_kernel<Op, float>), grid, dim3(kBlock), 0, s, p);
  else
    hipLaunchKernelGGL((fwd_generic_kernel<Op, double>), grid, dim3(kBlock), 0, s, p);
  return hipGetLastError();
}

}  // namespace bd

// Defines the two extern launch functions of one op in the translation unit that uses it.
#define BD_DEFINE_OP(OPTYPE, IDENT)                                                                  \
  hipError_t bd_fwd_tiled_##IDENT(int dt, int vec, const bd::FwdTiledParams &p, dim3 g, hipStream_t s) { \
    return bd::launch_fwd_tiled<OPTYPE>(dt, vec, p, g, s);                                           \
  }                                                                                                  \
  hipError_t bd_fwd_generic_##IDENT(int dt, const bd::FwdGenericParams &p, dim3 g, hipStream_t s) {  \
    return bd::launch_fwd_generic<OPTYPE>(dt, p, g, s);                                              \
  }
