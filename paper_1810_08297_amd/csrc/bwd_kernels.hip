// Reverse step of a broadcast node (Table 1 of arXiv 1810.08297): multiply the upstream
// adjoints by the cached Jacobian planes and, for an argument that was expanded along some
// dims, sum over those dims.  Independent of the op.  One streaming pass reads every
// adjoint and plane exactly once; the reductions ride on it (wavefront butterflies, LDS,
// per-block partial sums) and a small second pass adds the per-block partials in a fixed
// order.  No atomics anywhere: results are bitwise reproducible.
#include <hip/hip_runtime.h>

#include "dual.h"
#include "fwd_kernels.h"  // load_vec / store_vec
#include "kparams.h"

namespace bd {

// ---- accumulators ----------------------------------------------------------------------
// fp32 data: products of two floats are exact in double; sums run in double.
// fp64 data: error-free products and sums (two-term compensated, as in a dot product
// evaluated in twice the working precision); hi + lo is rounded once at the end.
struct dd {
  double hi, lo;
};

BD_DEV void two_sum(double a, double b, double &s, double &err) {
#pragma clang fp contract(off)
  s = a + b;
  double bb = s - a;
  err = (a - (s - bb)) + (b - bb);
}

template <class T> struct acc_traits;
template <> struct acc_traits<float> {
  using type = double;
  static BD_DEV double zero() { return 0.0; }
  static BD_DEV void add_prod(double &a, float x, float y) { a = __builtin_fma((double)x, (double)y, a); }
  static BD_DEV void add(double &a, double b) { a += b; }
  static BD_DEV float fin(double a) { return (float)a; }
};
template <> struct acc_traits<double> {
  using type = dd;
  static BD_DEV dd zero() { return dd{0.0, 0.0}; }
  static BD_DEV void add_prod(dd &a, double x, double y) {
#pragma clang fp contract(off)
    double p = x * y;
    double e = __builtin_fma(x, y, -p);
    double s, err;
    two_sum(a.hi, p, s, err);
    a.hi = s;
    a.lo = a.lo + (err + e);
  }
  static BD_DEV void add(dd &a, dd b) {
#pragma clang fp contract(off)
    double s, err;
    two_sum(a.hi, b.hi, s, err);
    a.hi = s;
    a.lo = (a.lo + b.lo) + err;
  }
  static BD_DEV double fin(dd a) { return a.hi + a.lo; }
};

// sum_i adj_i * P_i for one element of a full-shape gradient, rounded once
// (rows beyond the real M hold zeros and add nothing)
template <class T, int MAXM, int VEC>
BD_DEV T wide_dot(const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC], int v) {
  double t = 0.0;
#pragma unroll
  for (int i = 0; i < MAXM; ++i) t = __builtin_fma((double)adj[i][v], (double)P[i][v], t);
  return (T)t;
}

// ---- cross-lane movement -------------------------------------------------------------------
// DPP controls (gfx9 encoding): quad_perm[1,0,3,2] = 0xB1, quad_perm[2,3,0,1] = 0x4E,
// row_half_mirror = 0x141, row_mirror = 0x140.  Every lane has a valid source in each.
template <int CTRL>
BD_DEV double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <int CTRL> BD_DEV double lane_move(double x) { return dpp_f64<CTRL>(x); }
template <int CTRL> BD_DEV dd lane_move(dd x) { return dd{dpp_f64<CTRL>(x.hi), dpp_f64<CTRL>(x.lo)}; }
BD_DEV double lane_xor(double x, int m) { return __shfl_xor(x, m, 64); }
BD_DEV dd lane_xor(dd x, int m) { return dd{__shfl_xor(x.hi, m, 64), __shfl_xor(x.lo, m, 64)}; }

// Butterfly sum over aligned groups of 2^log2w lanes (log2w <= 6).  All 64 lanes must be
// active.  Afterwards the first lane of every group holds the group's sum; the order of
// the additions is fixed by the lane numbers alone.
template <class T, class A>
BD_DEV A seg_reduce(A v, int log2w) {
  using AT = acc_traits<T>;
  if (log2w > 0) AT::add(v, lane_move<0xB1>(v));
  if (log2w > 1) AT::add(v, lane_move<0x4E>(v));
  if (log2w > 2) AT::add(v, lane_move<0x141>(v));
  if (log2w > 3) AT::add(v, lane_move<0x140>(v));
  if (log2w > 4) AT::add(v, lane_xor(v, 16));
  if (log2w > 5) AT::add(v, lane_xor(v, 32));
  return v;
}

// ---- tiled main pass -------------------------------------------------------------------------
// Same TY x TX lane arrangement as the forward kernel.  Per row step a lane loads the M
// adjoint vectors once and then, gradient by gradient, the M plane vectors; what happens to
// t_j = sum_i adj_i * P_ij depends on the gradient's class:
//   full     : stored at once
//   row sum  : summed over the lane's columns, butterfly over the row's lanes in the
//              wavefront, then (rows wider than a wavefront) one LDS cell per wavefront
//   col sum  : added to the lane's own LDS accumulators, combined over the block's rows at the end
//   all sum  : added to the lane's own LDS accumulator, block tree at the end
// A block writes a final gradient directly when it alone covers the reduced extent,
// otherwise its partial sum goes to the workspace for the second pass.
template <class T, int VEC, int MCT>
__global__ __launch_bounds__(kBlock) void bwd_tiled_kernel(const BwdTiledParams p) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  constexpr int MAXM = MCT > 0 ? MCT : BCAST_MAX_OUTS;
  extern __shared__ __align__(16) unsigned char smem[];
  A *lds_row = reinterpret_cast<A *>(smem + p.lds_row_off);
  A *lds_col = reinterpret_cast<A *>(smem + p.lds_col_off);
  A *lds_all = reinterpret_cast<A *>(smem + p.lds_all_off);

  const int M = MCT > 0 ? MCT : p.M;
  const int tid = threadIdx.x;
  const int ltx = p.log2_tx;
  const int TX = 1 << ltx;
  const int tx = tid & (TX - 1);
  const int ty = tid >> ltx;
  const int TY = kBlock >> ltx;
  const int txw = ltx < 6 ? ltx : 6;
  const int wpr = ltx > 6 ? (1 << (ltx - 6)) : 1;
  const int rows_pb = TY * p.steps;
  const uint32_t nct = (uint32_t)p.n_ct;
  const uint32_t rt = blockIdx.x / nct, ct = blockIdx.x - rt * nct;
  const int64_t c0 = ((((int64_t)ct) << ltx) + tx) * VEC;
  const bool colvalid = c0 < p.C;
  const int64_t r0 = (int64_t)rt * rows_pb;
  const bool nt = p.nt_store != 0;

  for (int s = 0; s < p.n_col_slots; ++s)
#pragma unroll
    for (int v = 0; v < VEC; ++v) lds_col[(s * kBlock + tid) * VEC + v] = AT::zero();
  for (int s = 0; s < p.n_all_slots; ++s) lds_all[s * kBlock + tid] = AT::zero();

  for (int k = 0; k < p.steps; ++k) {
    const int ri = k * TY + ty;
    const int64_t r = r0 + ri;
    const bool valid = colvalid && r < p.R;
    T adj[MAXM][VEC];
#pragma unroll
    for (int i = 0; i < MAXM; ++i) {
      if (i < M && valid) {
        load_vec<T, VEC>(static_cast<const T *>(p.adj[i].p) + r * p.adj[i].sr + c0, adj[i]);
      } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) adj[i][v] = T(0);
      }
    }
    for (int e = 0; e < p.n_entries; ++e) {
      const BwdEntry &en = p.e[e];
      T P[MAXM][VEC];
#pragma unroll
      for (int i = 0; i < MAXM; ++i) {
        if (i < M && valid && en.P[i].p != nullptr) {
          load_vec<T, VEC>(static_cast<const T *>(en.P[i].p) + r * en.P[i].sr + c0, P[i]);
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) P[i][v] = T(0);
        }
      }
      if (en.cls == kGradFull) {
        if (valid) {
          T o[VEC];
#pragma unroll
          for (int v = 0; v < VEC; ++v) o[v] = wide_dot<T, MAXM, VEC>(adj, P, v);
          store_vec<T, VEC>(static_cast<T *>(en.g.p) + r * en.g.sr + c0, o, nt);
        }
      } else if (en.cls == kGradRowSum) {
        A rs = AT::zero();
#pragma unroll
        for (int v = 0; v < VEC; ++v)
#pragma unroll
          for (int i = 0; i < MAXM; ++i) AT::add_prod(rs, adj[i][v], P[i][v]);
        rs = seg_reduce<T, A>(rs, txw);
        if (ltx <= 6) {
          if (tx == 0 && r < p.R) {
            if (en.direct)
              static_cast<T *>(en.g.p)[r * en.g.sr] = AT::fin(rs);
            else
              reinterpret_cast<A *>(p.ws + en.ws_off)[r * p.n_ct + ct] = rs;
          }
        } else if ((tid & 63) == 0) {
          lds_row[(en.slot * rows_pb + ri) * wpr + (tx >> 6)] = rs;
        }
      } else if (en.cls == kGradColSum) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          A c = lds_col[(en.slot * kBlock + tid) * VEC + v];
#pragma unroll
          for (int i = 0; i < MAXM; ++i) AT::add_prod(c, adj[i][v], P[i][v]);
          lds_col[(en.slot * kBlock + tid) * VEC + v] = c;
        }
      } else if (en.cls == kGradAllSum) {
        A c = lds_all[en.slot * kBlock + tid];
#pragma unroll
        for (int v = 0; v < VEC; ++v)
#pragma unroll
          for (int i = 0; i < MAXM; ++i) AT::add_prod(c, adj[i][v], P[i][v]);
        lds_all[en.slot * kBlock + tid] = c;
      }
    }
  }
  if (p.n_row_slots + p.n_col_slots + p.n_all_slots == 0) return;
  __syncthreads();

  for (int e = 0; e < p.n_entries; ++e) {
    const BwdEntry &en = p.e[e];
    if (en.cls == kGradRowSum && ltx > 6) {
      for (int q = tid; q < rows_pb; q += kBlock) {
        const int64_t r = r0 + q;
        if (r < p.R) {
          A s = lds_row[(en.slot * rows_pb + q) * wpr];
          for (int w = 1; w < wpr; ++w) AT::add(s, lds_row[(en.slot * rows_pb + q) * wpr + w]);
          if (en.direct)
            static_cast<T *>(en.g.p)[r * en.g.sr] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[r * p.n_ct + ct] = s;
        }
      }
    } else if (en.cls == kGradColSum) {
      if (ty == 0 && colvalid) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          A s = lds_col[(en.slot * kBlock + tx) * VEC + v];
          for (int y = 1; y < TY; ++y) AT::add(s, lds_col[(en.slot * kBlock + y * TX + tx) * VEC + v]);
          if (en.direct)
            static_cast<T *>(en.g.p)[(c0 + v) * en.g.sc] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[(int64_t)rt * p.C + c0 + v] = s;
        }
      }
    } else if (en.cls == kGradAllSum) {
      A s = lds_all[en.slot * kBlock + tid];
      s = seg_reduce<T, A>(s, 6);
      __syncthreads();
      if ((tid & 63) == 0) lds_all[en.slot * kBlock + (tid >> 6)] = s;
      __syncthreads();
      if (tid == 0) {
        A t = lds_all[en.slot * kBlock];
        for (int w = 1; w < kBlock / 64; ++w) AT::add(t, lds_all[en.slot * kBlock + w]);
        if (en.direct)
          static_cast<T *>(en.g.p)[0] = AT::fin(t);
        else
          reinterpret_cast<A *>(p.ws + en.ws_off)[blockIdx.x] = t;
      }
    }
  }
}

// ---- second pass: add the per-block partial sums in a fixed order ------------------------------
template <class T>
__global__ __launch_bounds__(kBlock) void bwd_pass2_kernel(const Pass2Params p) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  __shared__ A sh[kBlock];
  int j = 0;
  for (int q = 1; q < p.n_jobs; ++q)
    if ((int64_t)blockIdx.x >= p.job[q].first_block) j = q;
  const Pass2Job &job = p.job[j];
  const int64_t b = (int64_t)blockIdx.x - job.first_block;
  const A *ws = reinterpret_cast<const A *>(p.ws + job.ws_off);
  T *g = static_cast<T *>(job.g);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (job.kind == 0) {  // one wavefront per output
    const int64_t out = b * (kBlock / 64) + wave;
    if (out < job.n_out) {
      A s = AT::zero();
      for (int64_t q = lane; q < job.n_part; q += 64) AT::add(s, ws[out * job.out_stride + q * job.part_stride]);
      s = seg_reduce<T, A>(s, 6);
      if (lane == 0) g[out * job.g_stride] = AT::fin(s);
    }
  } else if (job.kind == 1) {  // one block per output
    const int64_t out = b;
    A s = AT::zero();
    for (int64_t q = tid; q < job.n_part; q += kBlock) AT::add(s, ws[out * job.out_stride + q * job.part_stride]);
    s = seg_reduce<T, A>(s, 6);
    if (lane == 0) sh[wave] = s;
    __syncthreads();
    if (tid == 0) {
      A t = sh[0];
      for (int w = 1; w < kBlock / 64; ++w) AT::add(t, sh[w]);
      g[out * job.g_stride] = AT::fin(t);
    }
  } else {  // 64 adjacent outputs x 4 interleaved groups of partials
    const int64_t out = b * 64 + lane;
    A s = AT::zero();
    if (out < job.n_out)
      for (int64_t q = wave; q < job.n_part; q += kBlock / 64)
        AT::add(s, ws[out * job.out_stride + q * job.part_stride]);
    sh[tid] = s;
    __syncthreads();
    if (wave == 0 && out < job.n_out) {
      A t = sh[lane];
      for (int w = 1; w < kBlock / 64; ++w) AT::add(t, sh[w * 64 + lane]);
      g[out * job.g_stride] = AT::fin(t);
    }
  }
}

// ---- generic strided kernels: one gradient per launch ----------------------------------------------
template <class T>
__global__ __launch_bounds__(kBlock) void bwd_generic_full_kernel(const BwdGenericParams p) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= p.E) return;
  int64_t idx[BCAST_MAX_DIMS] = {0, 0, 0, 0};
  int64_t rem = e;
#pragma unroll
  for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
    if (d < p.nd) {
      idx[d] = rem % p.shape[d];
      rem /= p.shape[d];
    }
  auto off = [&](const GView &g) {
    int64_t o = 0;
#pragma unroll
    for (int d = 0; d < BCAST_MAX_DIMS; ++d) o += idx[d] * g.s[d];
    return o;
  };
  T a[BCAST_MAX_OUTS][1], P[BCAST_MAX_OUTS][1];
#pragma unroll
  for (int i = 0; i < BCAST_MAX_OUTS; ++i) {
    a[i][0] = (i < p.M) ? static_cast<const T *>(p.adj[i].p)[off(p.adj[i])] : T(0);
    P[i][0] = (i < p.M && p.P[i].p) ? static_cast<const T *>(p.P[i].p)[off(p.P[i])] : T(0);
  }
  static_cast<T *>(p.g.p)[off(p.g)] = wide_dot<T, BCAST_MAX_OUTS, 1>(a, P, 0);
}

// one block per gradient element; the block walks that element's fibre (the dims the
// argument was expanded along) with a fixed lane-to-term assignment
template <class T>
__global__ __launch_bounds__(kBlock) void bwd_generic_reduce_kernel(const BwdGenericParams p) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  __shared__ A sh[kBlock / 64];
  int64_t idx[BCAST_MAX_DIMS] = {0, 0, 0, 0};
  int64_t rem = blockIdx.x;
  for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
    if (d < p.nd && !p.reduced[d]) {
      idx[d] = rem % p.shape[d];
      rem /= p.shape[d];
    }
  int64_t goff = 0;
  for (int d = 0; d < BCAST_MAX_DIMS; ++d) goff += idx[d] * p.g.s[d];
  A s = AT::zero();
  for (int64_t q = threadIdx.x; q < p.n_fibre; q += kBlock) {
    int64_t rq = q;
    for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
      if (d < p.nd && p.reduced[d]) {
        idx[d] = rq % p.shape[d];
        rq /= p.shape[d];
      }
    for (int i = 0; i < p.M; ++i) {
      if (p.P[i].p == nullptr) continue;
      int64_t oa = 0, op = 0;
      for (int d = 0; d < BCAST_MAX_DIMS; ++d) {
        oa += idx[d] * p.adj[i].s[d];
        op += idx[d] * p.P[i].s[d];
      }
      AT::add_prod(s, static_cast<const T *>(p.adj[i].p)[oa], static_cast<const T *>(p.P[i].p)[op]);
    }
  }
  s = seg_reduce<T, A>(s, 6);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    A t = sh[0];
    for (int w = 1; w < kBlock / 64; ++w) AT::add(t, sh[w]);
    static_cast<T *>(p.g.p)[goff] = AT::fin(t);
  }
}

// ---- streaming copy with the tiled kernels' access pattern ------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kBlock) void copy_probe_kernel(f32x4 *__restrict__ dst,
                                                           const f32x4 *__restrict__ src, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n16) __builtin_nontemporal_store(src[i], &dst[i]);
}

}  // namespace bd

// ---- launch wrappers --------------------------------------------------------------------------------
using namespace bd;

hipError_t bd_bwd_tiled(int dt, int vec, const BwdTiledParams &p, dim3 grid, size_t lds, hipStream_t s) {
#define BD_LAUNCH(T, V)                                                                          \
  do {                                                                                           \
    if (p.M == 1)                                                                                \
      hipLaunchKernelGGL((bwd_tiled_kernel<T, V, 1>), grid, dim3(kBlock), lds, s, p);            \
    else if (p.M == 2)                                                                           \
      hipLaunchKernelGGL((bwd_tiled_kernel<T, V, 2>), grid, dim3(kBlock), lds, s, p);            \
    else                                                                                         \
      hipLaunchKernelGGL((bwd_tiled_kernel<T, V, 0>), grid, dim3(kBlock), lds, s, p);            \
  } while (0)
  if (dt == BCAST_F32) {
    if (vec > 1) BD_LAUNCH(float, 4); else BD_LAUNCH(float, 1);
  } else {
    if (vec > 1) BD_LAUNCH(double, 2); else BD_LAUNCH(double, 1);
  }
#undef BD_LAUNCH
  return hipGetLastError();
}

hipError_t bd_bwd_pass2(int dt, const Pass2Params &p, int64_t n_blocks, hipStream_t s) {
  if (dt == BCAST_F32)
    hipLaunchKernelGGL((bwd_pass2_kernel<float>), dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
  else
    hipLaunchKernelGGL((bwd_pass2_kernel<double>), dim3((unsigned)n_blocks), dim3(kBlock), 0, s, p);
  return hipGetLastError();
}

hipError_t bd_bwd_generic(int dt, bool reduce, const BwdGenericParams &p, int64_t n_blocks, hipStream_t s) {
  dim3 grid((unsigned)n_blocks);
  if (dt == BCAST_F32) {
    if (reduce) hipLaunchKernelGGL((bwd_generic_reduce_kernel<float>), grid, dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((bwd_generic_full_kernel<float>), grid, dim3(kBlock), 0, s, p);
  } else {
    if (reduce) hipLaunchKernelGGL((bwd_generic_reduce_kernel<double>), grid, dim3(kBlock), 0, s, p);
    else hipLaunchKernelGGL((bwd_generic_full_kernel<double>), grid, dim3(kBlock), 0, s, p);
  }
  return hipGetLastError();
}

hipError_t bd_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t s) {
  const int64_t n16 = (int64_t)(bytes / 16);
  if (n16 == 0) return hipSuccess;
  const int64_t blocks = (n16 + kBlock - 1) / kBlock;
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s,
                     static_cast<f32x4 *>(dst), static_cast<const f32x4 *>(src), n16);
  return hipGetLastError();
}
