// Unfused comparison system: the same scalar functions evaluated as a chain of whole-array
// primitives -- one kernel per primitive, every branch computed for every element and chosen
// with a select -- and differentiated by plain reverse mode, primitive by primitive (the kind of
// program the reverse-mode implementations of Sec. 3.2.1 and 3.2.2 of arXiv 1810.08297 run: each
// primitive of the cell update becomes a kernel of its own, with temporaries in memory between
// them).  It is NOT on the product path: it exists to be timed beside the fused dual-number
// kernels and is checked against the same oracle.
//
// Every array is contiguous, row major, [rows x cols]; an operand is a full array, a row vector
// [1 x cols], a column vector [rows x 1] or a scalar.  Temporaries are full arrays in the caller's
// workspace.  Masks are arrays of 0.0 / 1.0 in the value type.  Sums run in double.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include "bcast_dual.h"

namespace bd {
namespace unfused {

constexpr int kThreads = 256;

struct Operand {
  const void *p;
  int kind;  // BCAST_UNFUSED_FULL, _ROW_VECTOR, _COL_VECTOR, _SCALAR
};

// element (r, c .. c + V - 1) of an operand
template <class T, int V>
__device__ __forceinline__ void fetch(const Operand &a, int64_t r, int64_t c, int64_t C, T (&x)[V]) {
  const T *p = static_cast<const T *>(a.p);
  if (a.kind == BCAST_UNFUSED_FULL || a.kind == BCAST_UNFUSED_ROW_VECTOR) {
    const T *q = p + (a.kind == BCAST_UNFUSED_FULL ? r * C : 0) + c;
    if constexpr (V == 4 && sizeof(T) == 4) {
      const float4 v = *reinterpret_cast<const float4 *>(q);
      x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else if constexpr (V == 2 && sizeof(T) == 8) {
      const double2 v = *reinterpret_cast<const double2 *>(q);
      x[0] = v.x; x[1] = v.y;
    } else {
#pragma unroll
      for (int k = 0; k < V; ++k) x[k] = q[k];
    }
  } else {
    const T s = p[a.kind == BCAST_UNFUSED_COL_VECTOR ? r : 0];
#pragma unroll
    for (int k = 0; k < V; ++k) x[k] = s;
  }
}
template <class T, int V>
__device__ __forceinline__ void put(T *out, int64_t r, int64_t c, int64_t C, const T (&x)[V]) {
  T *q = out + r * C + c;
  if constexpr (V == 4 && sizeof(T) == 4) {
    *reinterpret_cast<float4 *>(q) = make_float4(x[0], x[1], x[2], x[3]);
  } else if constexpr (V == 2 && sizeof(T) == 8) {
    *reinterpret_cast<double2 *>(q) = make_double2(x[0], x[1]);
  } else {
#pragma unroll
    for (int k = 0; k < V; ++k) q[k] = x[k];
  }
}

// the primitives: out = f(a [, b [, m]])
enum Prim : int {
  kAdd, kSub, kMul, kNeg, kOneMinus, kSigmoid, kTanh, kExp, kLog1p, kEqConst, kGreater, kSelect,  // forward
  kSigmoidBwd,  // g * y * (1 - y)      (a = g, b = y = sigmoid(x))
  kTanhBwd,     // g * (1 - y * y)      (a = g, b = y = tanh(x))
  kExpBwd,      // g * y                (a = g, b = y = exp(x))  -- a plain mul; kept apart for the kernel count's sake
  kLog1pBwd,    // g / (1 + x)          (a = g, b = x)
};
template <class T> __device__ __forceinline__ T sigmoid_of(T x) { return T(1) / (T(1) + exp(-x)); }

template <class T, int V, int PRIM>
__global__ __launch_bounds__(kThreads) void prim_kernel(T *out, Operand a, Operand b, Operand m, T konst, int64_t R, int64_t C) {
  const int64_t per_row = C / V;
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= R * per_row) return;
  const int64_t r = idx / per_row, c = (idx - r * per_row) * V;
  T x[V], y[V], z[V], o[V];
  fetch<T, V>(a, r, c, C, x);
  if constexpr (PRIM == kAdd || PRIM == kSub || PRIM == kMul || PRIM == kGreater || PRIM == kSelect || PRIM >= kSigmoidBwd) fetch<T, V>(b, r, c, C, y);
  if constexpr (PRIM == kSelect) fetch<T, V>(m, r, c, C, z);
#pragma unroll
  for (int k = 0; k < V; ++k) {
    if constexpr (PRIM == kAdd) o[k] = x[k] + y[k];
    else if constexpr (PRIM == kSub) o[k] = x[k] - y[k];
    else if constexpr (PRIM == kMul || PRIM == kExpBwd) o[k] = x[k] * y[k];
    else if constexpr (PRIM == kNeg) o[k] = -x[k];
    else if constexpr (PRIM == kOneMinus) o[k] = T(1) - x[k];
    else if constexpr (PRIM == kSigmoid) o[k] = sigmoid_of(x[k]);
    else if constexpr (PRIM == kTanh) o[k] = tanh(x[k]);
    else if constexpr (PRIM == kExp) o[k] = exp(x[k]);
    else if constexpr (PRIM == kLog1p) o[k] = log1p(x[k]);
    else if constexpr (PRIM == kEqConst) o[k] = x[k] == konst ? T(1) : T(0);
    else if constexpr (PRIM == kGreater) o[k] = x[k] > y[k] ? T(1) : T(0);
    else if constexpr (PRIM == kSelect) o[k] = z[k] != T(0) ? x[k] : y[k];  // m ? a : b
    else if constexpr (PRIM == kSigmoidBwd) o[k] = x[k] * y[k] * (T(1) - y[k]);
    else if constexpr (PRIM == kTanhBwd) o[k] = x[k] * (T(1) - y[k] * y[k]);
    else if constexpr (PRIM == kLog1pBwd) o[k] = x[k] / (T(1) + y[k]);
  }
  put<T, V>(out, r, c, C, o);
}

// clears small buffers (a memset recorded into a captured graph has replayed wrongly; a kernel has not)
template <class T>
__global__ __launch_bounds__(kThreads) void fill_kernel(T *p, int64_t n, T value) {
  const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k < n) p[k] = value;
}

// ---- reductions of a full-shape gradient to a broadcast argument's shape (fixed order, no atomics) ----
__device__ __forceinline__ double block_sum(double v, double *sh) {
  const int tid = threadIdx.x;
  sh[tid] = v;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if (tid < s) sh[tid] += sh[tid + s];
    __syncthreads();
  }
  return sh[0];
}
// one block per row: out[r] = sum_c g[r, c]   (out: T, or double partials for the full sum)
template <class T, class O>
__global__ __launch_bounds__(kThreads) void row_sum_kernel(O *out, const T *g, int64_t R, int64_t C) {
  __shared__ double sh[kThreads];
  const int64_t r = blockIdx.x;
  double s = 0.0;
  for (int64_t c = threadIdx.x; c < C; c += kThreads) s += (double)g[r * C + c];
  s = block_sum(s, sh);
  if (threadIdx.x == 0) out[r] = (O)s;
}
// column sums in two stages: partial[chunk, c] over a chunk of rows, then the chunks in order
template <class T>
__global__ __launch_bounds__(kThreads) void col_partial_kernel(double *partial, const T *g, int64_t R, int64_t C, int64_t rows_per_chunk) {
  const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (c >= C) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk, r1 = r0 + rows_per_chunk < R ? r0 + rows_per_chunk : R;
  double s = 0.0;
  for (int64_t r = r0; r < r1; ++r) s += (double)g[r * C + c];
  partial[(int64_t)blockIdx.y * C + c] = s;
}
template <class T>
__global__ __launch_bounds__(kThreads) void col_final_kernel(T *out, const double *partial, int64_t C, int64_t n_chunks) {
  const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (c >= C) return;
  double s = 0.0;
  for (int64_t k = 0; k < n_chunks; ++k) s += partial[k * C + c];
  out[c] = (T)s;
}
template <class T>
__global__ __launch_bounds__(kThreads) void all_final_kernel(T *out, const double *row_sums, int64_t R) {
  __shared__ double sh[kThreads];
  double s = 0.0;
  for (int64_t r = threadIdx.x; r < R; r += kThreads) s += row_sums[r];
  s = block_sum(s, sh);
  if (threadIdx.x == 0) out[0] = (T)s;
}

// ---- the host side: a straight-line program of primitives over temporaries in the workspace ----------
template <class T>
struct Program {
  int64_t R, C, E;
  hipStream_t stream;
  unsigned char *ws;
  size_t ws_bytes, used = 0;
  int n_kernels = 0;
  bool failed = false;
  static constexpr int V = 16 / sizeof(T);

  void *take(size_t bytes) {
    bytes = (bytes + 255) & ~(size_t)255;
    if (used + bytes > ws_bytes) { failed = true; return ws; }
    void *p = ws + used;
    used += bytes;
    return p;
  }
  Operand temp() { return Operand{take((size_t)E * sizeof(T)), BCAST_UNFUSED_FULL}; }
  void fill(void *p, int64_t n, T value) {
    if (failed || n <= 0) return;
    hipLaunchKernelGGL((fill_kernel<T>), dim3((unsigned)((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, static_cast<T *>(p), n, value);
    ++n_kernels;
  }
  Operand zero_scalar() {
    void *p = take(256);
    fill(p, 1, T(0));
    return Operand{p, BCAST_UNFUSED_SCALAR};
  }

  template <int PRIM>
  Operand run(Operand out, Operand a, Operand b = Operand{nullptr, BCAST_UNFUSED_SCALAR}, Operand m = Operand{nullptr, BCAST_UNFUSED_SCALAR}, T konst = T(0)) {
    if (failed) return out;
    const bool vec = C % V == 0;
    const int64_t lanes = vec ? E / V : E;
    const dim3 grid((unsigned)((lanes + kThreads - 1) / kThreads));
    if (vec)
      hipLaunchKernelGGL((prim_kernel<T, V, PRIM>), grid, dim3(kThreads), 0, stream, static_cast<T *>(const_cast<void *>(out.p)), a, b, m, konst, R, C);
    else
      hipLaunchKernelGGL((prim_kernel<T, 1, PRIM>), grid, dim3(kThreads), 0, stream, static_cast<T *>(const_cast<void *>(out.p)), a, b, m, konst, R, C);
    ++n_kernels;
    return out;
  }
  template <int PRIM> Operand op(Operand a, Operand b = Operand{nullptr, BCAST_UNFUSED_SCALAR}) { return run<PRIM>(temp(), a, b); }
  template <int PRIM> Operand op_into(void *out, Operand a, Operand b = Operand{nullptr, BCAST_UNFUSED_SCALAR}) {
    return run<PRIM>(Operand{out, BCAST_UNFUSED_FULL}, a, b);
  }
  Operand eq_const(Operand a, T k) { return run<kEqConst>(temp(), a, Operand{nullptr, 0}, Operand{nullptr, 0}, k); }
  Operand select(Operand m, Operand a, Operand b) { return run<kSelect>(temp(), a, b, m); }
  Operand select_into(void *out, Operand m, Operand a, Operand b) { return run<kSelect>(Operand{out, BCAST_UNFUSED_FULL}, a, b, m); }

  // gradient of a broadcast argument from the full-shape gradient `g`
  void reduce_into(void *out, int kind, Operand g) {
    if (failed) return;
    const T *gp = static_cast<const T *>(g.p);
    if (kind == BCAST_UNFUSED_COL_VECTOR) {
      hipLaunchKernelGGL((row_sum_kernel<T, T>), dim3((unsigned)R), dim3(kThreads), 0, stream, static_cast<T *>(out), gp, R, C);
      ++n_kernels;
    } else if (kind == BCAST_UNFUSED_ROW_VECTOR) {
      const int64_t n_chunks = R < 64 ? 1 : (R / 64 < 64 ? R / 64 : 64), rows_per_chunk = (R + n_chunks - 1) / n_chunks;
      double *partial = static_cast<double *>(take((size_t)n_chunks * C * sizeof(double)));
      if (failed) return;
      const dim3 grid((unsigned)((C + kThreads - 1) / kThreads), (unsigned)n_chunks);
      hipLaunchKernelGGL((col_partial_kernel<T>), grid, dim3(kThreads), 0, stream, partial, gp, R, C, rows_per_chunk);
      hipLaunchKernelGGL((col_final_kernel<T>), dim3(grid.x), dim3(kThreads), 0, stream, static_cast<T *>(out), partial, C, n_chunks);
      n_kernels += 2;
    } else {  // scalar
      double *rows = static_cast<double *>(take((size_t)R * sizeof(double)));
      if (failed) return;
      hipLaunchKernelGGL((row_sum_kernel<T, double>), dim3((unsigned)R), dim3(kThreads), 0, stream, rows, gp, R, C);
      hipLaunchKernelGGL((all_final_kernel<T>), dim3(1), dim3(kThreads), 0, stream, static_cast<T *>(out), rows, R);
      n_kernels += 2;
    }
  }
  // a gradient goes to its destination directly when the argument has the full shape, else through a reduction
  void *grad_target(void *dst, int kind) { return kind == BCAST_UNFUSED_FULL ? dst : const_cast<void *>(temp().p); }
  void finish_grad(void *dst, int kind, void *computed) {
    if (kind != BCAST_UNFUSED_FULL) reduce_into(dst, kind, Operand{computed, BCAST_UNFUSED_FULL});
  }
};

// temporaries (full arrays) and reduction scratch each op's program takes, as an upper bound
inline size_t workspace_bytes(int which, size_t es, int64_t R, int64_t C) {
  const size_t plane = (((size_t)R * C * es) + 255) & ~(size_t)255;
  const int planes = which == 0 ? 48 : which == 1 ? 24 : which == 2 ? 8 : 28;
  return planes * plane + 8 * ((size_t)(64 * C + R) * sizeof(double) + 512);
}

// HM-LSTM cell update with hidden state and biases: args f i o g c h z z_below b_f b_i b_o b_g -> (c', h')
template <class T>
void hmlstm_update(Program<T> &P, const Operand *x, void *const *outs, const void *const *adj, void *const *grads, const int32_t *kind, bool with_h) {
  // with_h = false: the paper's six-argument update (c f i g z1 z2 -> c'), passed in as x = {f, i, -, g, c, -, z1, z2}
  const Operand f = x[0], i = x[1], o = x[2], g = x[3], c = x[4], h = x[5], z = x[6], zb = x[7];
  Operand F = f, I = i, O = o, G = g;
  if (with_h) {
    F = P.template op<kAdd>(f, x[8]);
    I = P.template op<kAdd>(i, x[9]);
    O = P.template op<kAdd>(o, x[10]);
    G = P.template op<kAdd>(g, x[11]);
  }
  const Operand sF = P.template op<kSigmoid>(F), sI = P.template op<kSigmoid>(I), tG = P.template op<kTanh>(G);
  const Operand flushv = P.template op<kMul>(sI, tG);
  const Operand keep = P.template op<kMul>(sF, c);
  const Operand updv = P.template op<kAdd>(keep, flushv);
  const Operand m_flush = P.eq_const(z, T(1));
  const Operand m_copy = P.template op<kMul>(P.eq_const(z, T(0)), P.eq_const(zb, T(0)));  // z == 0 and z_below == 0 (excludes z == 1)
  const Operand inner = P.select(m_copy, c, updv);
  const Operand cn = P.select_into(outs[0], m_flush, flushv, inner);
  Operand sO{}, tc{};
  if (with_h) {
    sO = P.template op<kSigmoid>(O);
    tc = P.template op<kTanh>(cn);
    const Operand hv = P.template op<kMul>(sO, tc);
    P.select_into(outs[1], m_copy, h, hv);
  }
  // ---- reverse pass, primitive by primitive ----
  const Operand zero = P.zero_scalar();
  const Operand a_c{adj[0], BCAST_UNFUSED_FULL};
  Operand g_cn = a_c;
  // gradient slots: with_h: f i o g c h b_f b_i b_o b_g ; without: c f i g
  void *const G_f = grads[with_h ? 0 : 1], *const G_i = grads[with_h ? 1 : 2], *const G_g = grads[with_h ? 3 : 3], *const G_c = grads[with_h ? 4 : 0];
  Operand g_O{};
  if (with_h) {
    const Operand a_h{adj[1], BCAST_UNFUSED_FULL};
    P.select_into(grads[5], m_copy, a_h, zero);               // h' = select(copy, h, hv): d/dh
    const Operand g_hv = P.select(m_copy, zero, a_h);
    const Operand g_sO = P.template op<kMul>(g_hv, tc);       // hv = sO * tc
    const Operand g_tc = P.template op<kMul>(g_hv, sO);
    g_cn = P.template op<kAdd>(a_c, P.template op<kTanhBwd>(g_tc, tc));  // c' feeds h' through tanh
    g_O = P.template op_into<kSigmoidBwd>(grads[2], g_sO, sO);
  }
  const Operand g_flush1 = P.select(m_flush, g_cn, zero);     // c' = select(flush, flushv, inner)
  const Operand g_inner = P.select(m_flush, zero, g_cn);
  const Operand g_c1 = P.select(m_copy, g_inner, zero);       // inner = select(copy, c, updv)
  const Operand g_updv = P.select(m_copy, zero, g_inner);
  const Operand g_flushv = P.template op<kAdd>(g_flush1, g_updv);  // updv = keep + flushv
  const Operand g_sF = P.template op<kMul>(g_updv, c);        // keep = sF * c
  const Operand g_c2 = P.template op<kMul>(g_updv, sF);
  P.template op_into<kAdd>(G_c, g_c1, g_c2);
  const Operand g_sI = P.template op<kMul>(g_flushv, tG);     // flushv = sI * tG
  const Operand g_tG = P.template op<kMul>(g_flushv, sI);
  const Operand g_F = P.template op_into<kSigmoidBwd>(G_f, g_sF, sF);
  const Operand g_I = P.template op_into<kSigmoidBwd>(G_i, g_sI, sI);
  const Operand g_G = P.template op_into<kTanhBwd>(G_g, g_tG, tG);
  if (with_h) {  // the biases were added to the gates: their gradients are the gates' gradients summed over the batch
    P.reduce_into(grads[6], kind[8], g_F);
    P.reduce_into(grads[7], kind[9], g_I);
    P.reduce_into(grads[8], kind[10], g_O);
    P.reduce_into(grads[9], kind[11], g_G);
  }
}

// tanh(x*y + b)
template <class T>
void tanh_xy_b(Program<T> &P, const Operand *x, void *const *outs, const void *const *adj, void *const *grads, const int32_t *kind) {
  const Operand u = P.template op<kAdd>(P.template op<kMul>(x[0], x[1]), x[2]);
  const Operand y = P.template op_into<kTanh>(outs[0], u);
  // u = x*y + b: the gradient of u is the gradient of b before its reduction
  void *gu = P.grad_target(grads[2], kind[2]);
  const Operand g_u = P.template op_into<kTanhBwd>(gu, Operand{adj[0], BCAST_UNFUSED_FULL}, y);
  void *gx = P.grad_target(grads[0], kind[0]), *gy = P.grad_target(grads[1], kind[1]);
  P.template op_into<kMul>(gx, g_u, x[1]);
  P.template op_into<kMul>(gy, g_u, x[0]);
  P.finish_grad(grads[0], kind[0], gx);
  P.finish_grad(grads[1], kind[1], gy);
  P.finish_grad(grads[2], kind[2], gu);
}

// exp(-A)*B + r if A + s > t else log1p(A*A)*r - s
template <class T>
void branchy5(Program<T> &P, const Operand *x, void *const *outs, const void *const *adj, void *const *grads, const int32_t *kind) {
  const Operand A = x[0], B = x[1], r = x[2], s = x[3], t = x[4];
  const Operand e = P.template op<kExp>(P.template op<kNeg>(A));
  const Operand y1 = P.template op<kAdd>(P.template op<kMul>(e, B), r);
  const Operand a2 = P.template op<kMul>(A, A);
  const Operand l = P.template op<kLog1p>(a2);
  const Operand y2 = P.template op<kSub>(P.template op<kMul>(l, r), s);
  const Operand mask = P.template op<kGreater>(P.template op<kAdd>(A, s), t);
  P.select_into(outs[0], mask, y1, y2);
  const Operand zero = P.zero_scalar();
  const Operand a_y{adj[0], BCAST_UNFUSED_FULL};
  const Operand g1 = P.select(mask, a_y, zero), g2 = P.select(mask, zero, a_y);
  // y1 = e*B + r: g_eB = g1, g_r += g1 ; e = exp(-A): g_A += -(g1 * B * e)
  const Operand g_e = P.template op<kMul>(g1, B);
  void *gB = P.grad_target(grads[1], kind[1]);
  P.template op_into<kMul>(gB, g1, e);
  P.finish_grad(grads[1], kind[1], gB);
  const Operand g_A1 = P.template op<kNeg>(P.template op<kExpBwd>(g_e, e));
  // y2 = l*r - s: g_l = g2 * r, g_r += g2 * l, g_s = -g2 ; l = log1p(a2): g_a2 = g_l / (1 + a2) ; a2 = A*A: g_A += 2 * g_a2 * A
  const Operand g_l = P.template op<kMul>(g2, r);
  void *gr = P.grad_target(grads[2], kind[2]);
  P.template op_into<kAdd>(gr, g1, P.template op<kMul>(g2, l));
  P.finish_grad(grads[2], kind[2], gr);
  const Operand g_a2 = P.template op<kLog1pBwd>(g_l, a2);
  const Operand g_A2h = P.template op<kMul>(g_a2, A);
  void *gA = P.grad_target(grads[0], kind[0]);
  P.template op_into<kAdd>(gA, g_A1, P.template op<kAdd>(g_A2h, g_A2h));
  P.finish_grad(grads[0], kind[0], gA);
  void *gs = P.grad_target(grads[3], kind[3]);
  P.template op_into<kNeg>(gs, g2);
  P.finish_grad(grads[3], kind[3], gs);
  // the threshold only appears in the predicate: no derivative reaches it
  P.fill(grads[4], kind[4] == BCAST_UNFUSED_FULL ? P.E : kind[4] == BCAST_UNFUSED_ROW_VECTOR ? P.C : kind[4] == BCAST_UNFUSED_COL_VECTOR ? P.R : 1, T(0));
}

template <class T>
int step(int which, int64_t R, int64_t C, int n_args, const void *const *args, const int32_t *kind, void *const *outs,
         const void *const *adj, void *const *grads, void *ws, size_t ws_bytes, hipStream_t stream, int32_t *n_kernels) {
  Program<T> P{R, C, R * C, stream, static_cast<unsigned char *>(ws), ws_bytes};
  Operand x[BCAST_MAX_ARGS];
  for (int j = 0; j < n_args; ++j) x[j] = Operand{args[j], kind[j]};
  (void)hipGetLastError();
  if (which == 0) {
    hmlstm_update<T>(P, x, outs, adj, grads, kind, true);
  } else if (which == 1) {  // c f i g z1 z2 -> the slots of the full update
    Operand y[12] = {x[1], x[2], Operand{nullptr, 0}, x[3], x[0], Operand{nullptr, 0}, x[4], x[5]};
    hmlstm_update<T>(P, y, outs, adj, grads, kind, false);
  } else if (which == 2) {
    tanh_xy_b<T>(P, x, outs, adj, grads, kind);
  } else {
    branchy5<T>(P, x, outs, adj, grads, kind);
  }
  if (n_kernels) *n_kernels = P.n_kernels;
  if (P.failed) return BCAST_ERR_WORKSPACE_TOO_SMALL;
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    std::fprintf(stderr, "bcast_dual: a launch of the unfused comparison failed: %s\n", hipGetErrorString(e));
    return BCAST_ERR_LAUNCH_FAILED;
  }
  return BCAST_OK;
}

}  // namespace unfused
}  // namespace bd

// which program an op name selects (-1: none)
static int unfused_program(int32_t op_id) {
  const char *name = bcast_op_name(op_id);
  if (name == nullptr) return -1;
  const char *known[] = {"hmlstm_update", "update_c", "tanh_xy_b", "branchy5"};
  for (int k = 0; k < 4; ++k)
    if (std::strcmp(name, known[k]) == 0) return k;
  return -1;
}

extern "C" {

size_t bcast_unfused_workspace(int32_t op_id, bcast_dtype dt, int64_t rows, int64_t cols) {
  const int which = unfused_program(op_id);
  if (which < 0 || (dt != BCAST_F32 && dt != BCAST_F64) || rows <= 0 || cols <= 0) return 0;
  return bd::unfused::workspace_bytes(which, dt == BCAST_F32 ? 4 : 8, rows, cols);
}

int bcast_unfused_step(int32_t op_id, bcast_dtype dt, int64_t rows, int64_t cols, int32_t n_args, const void *const *args,
                       const int32_t *arg_kind, int32_t n_out, void *const *outs, const void *const *adjoints, int32_t n_grads,
                       void *const *grads, void *workspace, size_t workspace_bytes, void *stream, int32_t *n_kernels) {
  const int which = unfused_program(op_id);
  if (op_id < 0 || op_id >= bcast_op_count()) return BCAST_ERR_INVALID_OP;
  if (which < 0) return BCAST_ERR_UNSUPPORTED;
  if (dt != BCAST_F32 && dt != BCAST_F64) return BCAST_ERR_BAD_DTYPE;
  int32_t na = 0, no = 0;
  uint32_t nondiff = 0;
  bcast_op_info(op_id, &na, &no, &nondiff, nullptr);
  if (n_args != na || n_out != no || n_grads != na - __builtin_popcount(nondiff)) return BCAST_ERR_BAD_ARG_COUNT;
  if (!args || !arg_kind || !outs || !adjoints || !grads) return BCAST_ERR_NULL_POINTER;
  if (rows < 0 || cols < 0 || rows > ((int64_t)1 << 31) - 1 || cols > ((int64_t)1 << 40) / (rows > 0 ? rows : 1)) return BCAST_ERR_SHAPE_MISMATCH;
  for (int j = 0; j < n_args; ++j) {
    if (arg_kind[j] < BCAST_UNFUSED_FULL || arg_kind[j] > BCAST_UNFUSED_SCALAR) return BCAST_ERR_SHAPE_MISMATCH;
    if (!args[j] && rows * cols > 0) return BCAST_ERR_NULL_POINTER;
  }
  // the programs read the update's gates, cell and hidden state as full arrays
  const int full_upto = which == 0 ? 6 : which == 1 ? 4 : which == 3 ? 2 : 0;
  for (int j = 0; j < full_upto; ++j)
    if (arg_kind[j] != BCAST_UNFUSED_FULL) return BCAST_ERR_UNSUPPORTED;
  for (int i = 0; i < n_out; ++i)
    if ((!outs[i] || !adjoints[i]) && rows * cols > 0) return BCAST_ERR_NULL_POINTER;
  for (int j = 0; j < n_grads; ++j)
    if (!grads[j] && rows * cols > 0) return BCAST_ERR_NULL_POINTER;
  if (rows * cols == 0) {
    if (n_kernels) *n_kernels = 0;
    return BCAST_OK;
  }
  if (workspace == nullptr) return BCAST_ERR_NULL_POINTER;
  if (workspace_bytes < bcast_unfused_workspace(op_id, dt, rows, cols)) return BCAST_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return BCAST_ERR_MISALIGNED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dt == BCAST_F32)
    return bd::unfused::step<float>(which, rows, cols, n_args, args, arg_kind, outs, adjoints, grads, workspace, workspace_bytes, s, n_kernels);
  return bd::unfused::step<double>(which, rows, cols, n_args, args, arg_kind, outs, adjoints, grads, workspace, workspace_bytes, s, n_kernels);
}

}  // extern "C"
