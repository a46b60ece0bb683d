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

// Sum over one whole wavefront (all 64 lanes active); every lane returns the total.  Four
// DPP butterfly steps give each 16-lane row its sum, the four row sums are then read through
// scalar registers and added in lane order.
BD_DEV double read_lane(double x, int lane) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), lane),
                          __builtin_amdgcn_readlane(__double2loint(x), lane));
}
BD_DEV dd read_lane(dd x, int lane) { return dd{read_lane(x.hi, lane), read_lane(x.lo, lane)}; }
template <class T, class A>
BD_DEV A wave_total(A v) {
  using AT = acc_traits<T>;
  v = seg_reduce<T, A>(v, 4);
  A t = read_lane(v, 0);
  AT::add(t, read_lane(v, 16));
  AT::add(t, read_lane(v, 32));
  AT::add(t, read_lane(v, 48));
  return t;
}

// ---- tiled main pass -------------------------------------------------------------------------
// Same TY x TX lane arrangement as the forward kernel, walking `steps` rows per block.  Per
// row step a lane loads the M adjoint vectors and the M plane vectors of every gradient;
// what happens to t_j = sum_i adj_i * P_ij depends on the gradient's class:
//   full     : stored at once
//   row sum  : summed over the lane's columns, reduced over the row's lanes in the
//              wavefront, then (rows wider than a wavefront) one LDS cell per wavefront
//   col sum  : added to the lane's own LDS accumulators, combined over the block's rows at the end
//   all sum  : added to the lane's own LDS accumulator, block tree at the end
// A block writes a final gradient directly when it alone covers the reduced extent,
// otherwise its partial sum goes to the workspace for the second pass.
//
// Two kernels share this scheme.  The signature kernel is compiled for a fixed number of
// outputs and of gradients of each class (the host sorts the gradient table by class), so
// every table access is a constant, all loads of a row step are issued before the first
// use and nothing is decided at run time but the ragged edge.  The generic kernel reads
// the class of each gradient from the table and takes any mix, one gradient at a time.
template <class T, int VEC>
struct BwdGeom {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  int tid, ltx, TX, tx, ty, TY, wpr, rows_pb;
  uint32_t bid, rt, ct;
  int64_t c0, r0;
  bool colvalid, interior;
  uint32_t off0, off_step;
  A *lds_row, *lds_col, *lds_all;

  BD_DEV BwdGeom(const BwdTiledParams &p, unsigned char *smem) {
    tid = threadIdx.x;
    ltx = p.log2_tx;
    TX = 1 << ltx;
    tx = tid & (TX - 1);
    ty = tid >> ltx;
    TY = kBlock >> ltx;
    wpr = ltx > 6 ? (1 << (ltx - 6)) : 1;
    rows_pb = TY * p.steps;
    const uint32_t nct = (uint32_t)p.n_ct;
    // In reverse mode the grid is walked from the last tile to the first: the planes that
    // the forward kernel wrote last are the ones still held by the memory-side cache.
    bid = p.reverse ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    rt = bid / nct;
    ct = bid - rt * nct;
    c0 = ((((int64_t)ct) << ltx) + tx) * VEC;
    colvalid = c0 < p.C;
    r0 = (int64_t)rt * rows_pb;
    interior = r0 + rows_pb <= p.R && ((((int64_t)ct + 1) << ltx) * VEC) <= p.C;
    // one byte offset per lane and row serves the adjoints, every plane and every full gradient
    off0 = (uint32_t)((r0 + ty) * p.row_stride + c0) * (uint32_t)sizeof(T);
    off_step = (uint32_t)(TY * p.row_stride) * (uint32_t)sizeof(T);
    lds_row = reinterpret_cast<A *>(smem + p.lds_row_off);
    lds_col = reinterpret_cast<A *>(smem + p.lds_col_off);
    lds_all = reinterpret_cast<A *>(smem + p.lds_all_off);
    for (int s = 0; s < p.n_col_slots; ++s)
#pragma unroll
      for (int v = 0; v < VEC; ++v) lds_col[(s * kBlock + tid) * VEC + v] = AT::zero();
    for (int s = 0; s < p.n_all_slots; ++s) lds_all[s * kBlock + tid] = AT::zero();
  }
};

// one vector of a plane; lanes outside the problem read offset 0 and get zeros
template <class T, int VEC, bool EDGE>
BD_DEV void load_plane(const void *base, uint32_t off, bool valid, T (&x)[VEC]) {
  if (EDGE) {
    load_vec<T, VEC>(at<const T>(base, valid ? off : 0u), x);
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = valid ? x[v] : T(0);
  } else {
    load_vec<T, VEC>(at<const T>(base, off), x);
  }
}

// the per-class treatment of one gradient at one row step
template <class T, int VEC, int MAXM, bool EDGE>
BD_DEV void apply_full(const BwdEntry &en, const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC], uint32_t off,
                       bool valid, bool nt) {
  T o[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) o[v] = wide_dot<T, MAXM, VEC>(adj, P, v);
  if (!EDGE || valid) store_vec<T, VEC>(at<T>(en.g.p, off), o, nt);
}
template <class T, int VEC, int MAXM>
BD_DEV void apply_rowsum(const BwdTiledParams &p, const BwdGeom<T, VEC> &g, const BwdEntry &en,
                         const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC], int64_t r, int ri) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  A rs = AT::zero();
#pragma unroll
  for (int v = 0; v < VEC; ++v)
#pragma unroll
    for (int i = 0; i < MAXM; ++i) AT::add_prod(rs, adj[i][v], P[i][v]);
  if (g.ltx >= 6) {  // the wavefront lies inside one row
    rs = wave_total<T, A>(rs);
    if ((g.tid & 63) == 0 && r < p.R) {
      if (g.ltx > 6)
        g.lds_row[(en.slot * g.rows_pb + ri) * g.wpr + (g.tx >> 6)] = rs;
      else if (en.direct)
        static_cast<T *>(en.g.p)[r * en.g.sr] = AT::fin(rs);
      else
        reinterpret_cast<A *>(p.ws + en.ws_off)[r * p.n_ct + g.ct] = rs;
    }
  } else {  // several rows per wavefront: segmented butterfly
    rs = seg_reduce<T, A>(rs, g.ltx);
    if (g.tx == 0 && r < p.R) {
      if (en.direct)
        static_cast<T *>(en.g.p)[r * en.g.sr] = AT::fin(rs);
      else
        reinterpret_cast<A *>(p.ws + en.ws_off)[r * p.n_ct + g.ct] = rs;
    }
  }
}
template <class T, int VEC, int MAXM>
BD_DEV void apply_colsum(const BwdGeom<T, VEC> &g, const BwdEntry &en, const T (&adj)[MAXM][VEC],
                         const T (&P)[MAXM][VEC]) {
  using AT = acc_traits<T>;
#pragma unroll
  for (int v = 0; v < VEC; ++v) {
    auto c = g.lds_col[(en.slot * kBlock + g.tid) * VEC + v];
#pragma unroll
    for (int i = 0; i < MAXM; ++i) AT::add_prod(c, adj[i][v], P[i][v]);
    g.lds_col[(en.slot * kBlock + g.tid) * VEC + v] = c;
  }
}
template <class T, int VEC, int MAXM>
BD_DEV void apply_allsum(const BwdGeom<T, VEC> &g, const BwdEntry &en, const T (&adj)[MAXM][VEC],
                         const T (&P)[MAXM][VEC]) {
  using AT = acc_traits<T>;
  auto c = g.lds_all[en.slot * kBlock + g.tid];
#pragma unroll
  for (int v = 0; v < VEC; ++v)
#pragma unroll
    for (int i = 0; i < MAXM; ++i) AT::add_prod(c, adj[i][v], P[i][v]);
  g.lds_all[en.slot * kBlock + g.tid] = c;
}

// after the row walk: combine what the block's lanes parked in LDS
template <class T, int VEC>
BD_DEV void bwd_finalize(const BwdTiledParams &p, const BwdGeom<T, VEC> &g) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  if (p.n_row_slots + p.n_col_slots + p.n_all_slots == 0) return;
  __syncthreads();
  for (int e = 0; e < p.n_entries; ++e) {
    const BwdEntry &en = p.e[e];
    if (en.cls == kGradRowSum && g.ltx > 6) {
      for (int q = g.tid; q < g.rows_pb; q += kBlock) {
        const int64_t r = g.r0 + q;
        if (r < p.R) {
          A s = g.lds_row[(en.slot * g.rows_pb + q) * g.wpr];
          for (int w = 1; w < g.wpr; ++w) AT::add(s, g.lds_row[(en.slot * g.rows_pb + q) * g.wpr + w]);
          if (en.direct)
            static_cast<T *>(en.g.p)[r * en.g.sr] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[r * p.n_ct + g.ct] = s;
        }
      }
    } else if (en.cls == kGradColSum) {
      if (g.ty == 0 && g.colvalid) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          A s = g.lds_col[(en.slot * kBlock + g.tx) * VEC + v];
          for (int y = 1; y < g.TY; ++y) AT::add(s, g.lds_col[(en.slot * kBlock + y * g.TX + g.tx) * VEC + v]);
          if (en.direct)
            static_cast<T *>(en.g.p)[(g.c0 + v) * en.g.sc] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[(int64_t)g.rt * p.C + g.c0 + v] = s;
        }
      }
    } else if (en.cls == kGradAllSum) {
      A s = g.lds_all[en.slot * kBlock + g.tid];
      s = wave_total<T, A>(s);
      __syncthreads();
      if ((g.tid & 63) == 0) g.lds_all[en.slot * kBlock + (g.tid >> 6)] = s;
      __syncthreads();
      if (g.tid == 0) {
        A t = g.lds_all[en.slot * kBlock];
        for (int w = 1; w < kBlock / 64; ++w) AT::add(t, g.lds_all[en.slot * kBlock + w]);
        if (en.direct)
          static_cast<T *>(en.g.p)[0] = AT::fin(t);
        else
          reinterpret_cast<A *>(p.ws + en.ws_off)[g.bid] = t;
      }
    }
  }
}

// Signature kernel: M outputs; the gradient table holds NF full, then NR row-sum, then NC
// col-sum, then NA all-sum gradients.  Bit e*M + i of ABSENT says that plane i of gradient e
// is absent (a structurally zero partial the caller chose not to store): it is neither
// loaded nor multiplied.
template <class T, int VEC, int M, int NF, int NR, int NC, int NA, uint64_t ABSENT>
__global__ __launch_bounds__(kBlock) void bwd_sig_kernel(const BwdTiledParams p) {
  constexpr int NE = NF + NR + NC + NA;
  extern __shared__ __align__(16) unsigned char smem[];
  const BwdGeom<T, VEC> g(p, smem);
  const bool nt = p.nt_store != 0;
  auto walk = [&](auto edge_tag) {
    constexpr bool EDGE = decltype(edge_tag)::value;
    uint32_t off = g.off0;
    for (int k = 0; k < p.steps; ++k, off += g.off_step) {
      const int ri = k * g.TY + g.ty;
      const int64_t r = g.r0 + ri;
      const bool valid = g.colvalid && r < p.R;
      T adj[M][VEC], P[NE][M][VEC];
#pragma unroll
      for (int i = 0; i < M; ++i) load_plane<T, VEC, EDGE>(p.adj[i].p, off, valid, adj[i]);
#pragma unroll
      for (int e = 0; e < NE; ++e)
#pragma unroll
        for (int i = 0; i < M; ++i) {
          if ((ABSENT >> (e * M + i)) & 1u) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) P[e][i][v] = T(0);
          } else {
            load_plane<T, VEC, EDGE>(p.e[e].P[i].p, off, valid, P[e][i]);
          }
        }
#pragma unroll
      for (int e = 0; e < NF; ++e) apply_full<T, VEC, M, EDGE>(p.e[e], adj, P[e], off, valid, nt);
#pragma unroll
      for (int e = NF; e < NF + NR; ++e) apply_rowsum<T, VEC, M>(p, g, p.e[e], adj, P[e], r, ri);
#pragma unroll
      for (int e = NF + NR; e < NF + NR + NC; ++e) apply_colsum<T, VEC, M>(g, p.e[e], adj, P[e]);
#pragma unroll
      for (int e = NF + NR + NC; e < NE; ++e) apply_allsum<T, VEC, M>(g, p.e[e], adj, P[e]);
    }
  };
  if (g.interior)
    walk(std::false_type{});
  else
    walk(std::true_type{});
  bwd_finalize<T, VEC>(p, g);
}

// Generic kernel: any number of outputs up to BCAST_MAX_OUTS (MCT = 0) and any mix of
// gradient classes and absent planes, one gradient at a time.
template <class T, int VEC, int MCT>
__global__ __launch_bounds__(kBlock) void bwd_tiled_kernel(const BwdTiledParams p) {
  constexpr int MAXM = MCT > 0 ? MCT : BCAST_MAX_OUTS;
  extern __shared__ __align__(16) unsigned char smem[];
  const BwdGeom<T, VEC> g(p, smem);
  const int M = MCT > 0 ? MCT : p.M;
  const bool nt = p.nt_store != 0;
  uint32_t off = g.off0;
  for (int k = 0; k < p.steps; ++k, off += g.off_step) {
    const int ri = k * g.TY + g.ty;
    const int64_t r = g.r0 + ri;
    const bool valid = g.colvalid && r < p.R;
    T adj[MAXM][VEC];
#pragma unroll
    for (int i = 0; i < MAXM; ++i) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) adj[i][v] = T(0);
      if (i < M) load_plane<T, VEC, true>(p.adj[i].p, off, valid, adj[i]);
    }
    for (int e = 0; e < p.n_entries; ++e) {
      const BwdEntry &en = p.e[e];
      T P[MAXM][VEC];
#pragma unroll
      for (int i = 0; i < MAXM; ++i) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) P[i][v] = T(0);
        if (i < M && en.P[i].p != nullptr) load_plane<T, VEC, true>(en.P[i].p, off, valid, P[i]);
      }
      if (en.cls == kGradFull)
        apply_full<T, VEC, MAXM, true>(en, adj, P, off, valid, nt);
      else if (en.cls == kGradRowSum)
        apply_rowsum<T, VEC, MAXM>(p, g, en, adj, P, r, ri);
      else if (en.cls == kGradColSum)
        apply_colsum<T, VEC, MAXM>(g, en, adj, P);
      else if (en.cls == kGradAllSum)
        apply_allsum<T, VEC, MAXM>(g, en, adj, P);
    }
  }
  bwd_finalize<T, VEC>(p, g);
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

// ---- streaming probe with the tiled kernels' access pattern --------------------------------------------
// Block b moves the b-th 4 KiB chunk of every plane: it reads n_in planes, adds them up and
// writes n_out planes.  Chunk b of plane k lives at base_k + b * stride_k (in floats), so the
// same kernel measures separate planes (stride 1024) and planes interleaved in one buffer.
struct ProbeParams {
  int32_t n_in, n_out;
  int64_t n_chunks;
  const float *in[32];
  int64_t in_stride[32];
  float *out[32];
  int64_t out_stride[32];
  float *sink;
};
typedef float f32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kBlock) void stream_probe_kernel(const ProbeParams p) {
  const int64_t b = blockIdx.x;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  int k = 0;
  for (; k + 8 <= p.n_in; k += 8) {  // eight loads in flight per lane
    f32x4 t[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
      t[q] = *reinterpret_cast<const f32x4 *>(p.in[k + q] + b * p.in_stride[k + q] + threadIdx.x * 4);
#pragma unroll
    for (int q = 0; q < 8; ++q) acc += t[q];
  }
  for (; k < p.n_in; ++k)
    acc += *reinterpret_cast<const f32x4 *>(p.in[k] + b * p.in_stride[k] + threadIdx.x * 4);
  for (int k = 0; k < p.n_out; ++k)
    __builtin_nontemporal_store(acc + (float)k, reinterpret_cast<f32x4 *>(p.out[k] + b * p.out_stride[k] + threadIdx.x * 4));
  if (p.n_out == 0 && acc[0] == 12345.678f) p.sink[0] = acc[1];  // keeps the loads alive
}

}  // namespace bd

// ---- launch wrappers --------------------------------------------------------------------------------
using namespace bd;

// Gradient-class signatures with a compiled kernel: {M, full, row-sum, col-sum, all-sum,
// absent-plane mask}.  The HM-LSTM update appears twice: with all 20 planes, and with the
// planes of c' with respect to o and h (and the bias b_o) left out -- they are zero on
// every branch.  Table order there: f i o g c h | b_f b_i b_o b_g, planes (c', h') per gradient.
#define BD_HM_LEAN ((1ull << (2 * 2 + 0)) | (1ull << (5 * 2 + 0)) | (1ull << (8 * 2 + 0)))
#define BD_SIGNATURES(X)                                          \
  X(2, 6, 4, 0, 0, 0ull) /* HM-LSTM update, per-row biases */     \
  X(2, 6, 4, 0, 0, BD_HM_LEAN)                                    \
  X(1, 2, 1, 0, 0, 0ull) /* tanh(x*y + b) */                      \
  X(1, 2, 1, 1, 1, 0ull) /* branchy5 */                           \
  X(1, 2, 1, 1, 1, 1ull << 4) /* branchy5 without the always-zero plane of t */ \
  X(1, 4, 0, 0, 0, 0ull) /* six-argument cell update */           \
  X(1, 1, 0, 0, 0, 0ull) X(1, 2, 0, 0, 0, 0ull) X(1, 3, 0, 0, 0, 0ull) X(1, 5, 0, 0, 0, 0ull) X(1, 8, 0, 0, 0, 0ull)

bool bd_bwd_has_signature(int M, int nf, int nr, int nc, int na, uint64_t absent) {
#define BD_SIG_TEST(m, f, r, c, a, ab) \
  if (M == m && nf == f && nr == r && nc == c && na == a && absent == (ab)) return true;
  BD_SIGNATURES(BD_SIG_TEST)
#undef BD_SIG_TEST
  return false;
}

hipError_t bd_bwd_tiled(int dt, int vec, bool signature, int nf, int nr, int nc, int na, uint64_t absent,
                        const BwdTiledParams &p, dim3 grid, size_t lds, hipStream_t s) {
  const bool widest = (dt == BCAST_F32 && vec == 4) || (dt == BCAST_F64 && vec == 2);
  if (signature && widest) {
#define BD_SIG_GO(m, f, r, c, a, ab)                                                                        \
  if (p.M == m && nf == f && nr == r && nc == c && na == a && absent == (ab)) {                             \
    if (dt == BCAST_F32)                                                                                    \
      hipLaunchKernelGGL((bwd_sig_kernel<float, 4, m, f, r, c, a, (ab)>), grid, dim3(kBlock), lds, s, p);   \
    else                                                                                                    \
      hipLaunchKernelGGL((bwd_sig_kernel<double, 2, m, f, r, c, a, (ab)>), grid, dim3(kBlock), lds, s, p);  \
    return hipGetLastError();                                                                               \
  }
    BD_SIGNATURES(BD_SIG_GO)
#undef BD_SIG_GO
  }
#define BD_GO(T, V, MM) hipLaunchKernelGGL((bwd_tiled_kernel<T, V, MM>), grid, dim3(kBlock), lds, s, p)
#define BD_LAUNCH(T, V)                \
  do {                                 \
    if (p.M == 1) BD_GO(T, V, 1);      \
    else if (p.M == 2) BD_GO(T, V, 2); \
    else BD_GO(T, V, 0);               \
  } while (0)
  if (dt == BCAST_F32) {
    if (vec == 4) BD_LAUNCH(float, 4);
    else if (vec == 2) BD_LAUNCH(float, 2);
    else BD_LAUNCH(float, 1);
  } else {
    if (vec == 2) BD_LAUNCH(double, 2);
    else BD_LAUNCH(double, 1);
  }
#undef BD_LAUNCH
#undef BD_GO
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

hipError_t bd_stream_probe(int n_in, const void *const *in, const int64_t *in_stride, int n_out, void *const *out,
                           const int64_t *out_stride, int64_t n_chunks, hipStream_t s) {
  ProbeParams p{};
  p.n_in = n_in;
  p.n_out = n_out;
  p.n_chunks = n_chunks;
  for (int k = 0; k < n_in; ++k) {
    p.in[k] = static_cast<const float *>(in[k]);
    p.in_stride[k] = in_stride[k];
  }
  for (int k = 0; k < n_out; ++k) {
    p.out[k] = static_cast<float *>(out[k]);
    p.out_stride[k] = out_stride[k];
  }
  p.sink = n_out > 0 ? p.out[0] : const_cast<float *>(p.in[0]);
#ifndef BD_PROBE_LDS
#define BD_PROBE_LDS 0
#endif
  hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)n_chunks), dim3(kBlock), BD_PROBE_LDS, s, p);
  return hipGetLastError();
}
