// Device-side building blocks of the reverse step (Table 1 of arXiv 1810.08297), shared by
// the backward kernels that read cached planes and by the recompute kernels that evaluate
// the dual numbers again: accumulators, cross-lane sums, the block geometry and the
// per-class treatment of one gradient.
#pragma once
#include <hip/hip_runtime.h>

#include "dual.h"
#include "fwd_kernels.h"  // load_vec / store_vec / at
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
  // an infinite or NaN sum keeps its high part: the error terms of the additions that met it are inf - inf
  static BD_DEV double fin(dd a) { return __builtin_isfinite(a.hi) ? a.hi + a.lo : a.hi; }
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
// use and nothing is decided at run time but the ragged edge.  The other kernel reads the
// class of each gradient from the table at run time and takes any mix, four gradients'
// planes in flight at a time.
template <class T, int VEC>
struct BwdGeom {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  int tid, ltx, TX, tx, ty, TY, wpr, rows_pb;
  uint32_t bid, rt, ct;  // bid: the block's index within its slice
  int64_t slice, O;      // the block's slice of a 3-D problem and the number of slices (0 and 1 for two dims)
  int64_t c0, r_first;  // r_first: row of the block's first row step at ty = 0
  int64_t r_step;       // rows from one row step of the block to its next
  bool colvalid, interior;
  int shift;              // ragged rows: columns by which the row's last lane moves its loads to the left (see unshift)
  uint32_t lane_uniform;  // (lane's row within a row step * common row stride + lane's first load column) * sizeof(T)
  uint32_t col_off;       // byte offset of the lane's first load column within a row
  int chunk_cols;        // columns one lane arrangement covers: TX * VEC
  uint32_t chunk_bytes;  // ... in bytes
  A *lds_row, *lds_col, *lds_all;

  BD_DEV BwdGeom(const BwdTiledParams &p, unsigned char *smem) {
    // the scalars at the head of the argument block and the grid size, fetched together (see arrived)
    const uint32_t grid = gridDim.x;
    arrived(low_word(p.R) ^ low_word(p.C) ^ low_word(p.log2_tx) ^ low_word(p.steps) ^ low_word(p.reverse) ^
            low_word(p.xcd_remap) ^ low_word(p.col_chunks) ^ low_word(p.interleave) ^ low_word(p.ragged) ^ low_word(p.n_col_slots) ^
            low_word(p.n_all_slots) ^ p.lds_row_off ^ p.lds_col_off ^ p.lds_all_off ^ low_word(p.n_ct) ^ low_word(p.n_rt) ^
            low_word(p.row_stride) ^ low_word(p.O) ^ low_word(p.tiles_per_slice) ^ low_word(p.outer_stride) ^ low_word(p.ws) ^ grid);
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
    bid = blockIdx.x;
    if (p.xcd_remap) bid = (bid & 7u) * (grid >> 3) + (bid >> 3);
    if (p.reverse == 1) {
      bid = grid - 1 - bid;
    } else if (p.reverse == 2) {
      // last to first in groups of eight, each block keeping its place within its group: the
      // hardware deals consecutive blocks round-robin to the 8 XCDs, so a tile then stays on the
      // XCD (its L2, its address-translation cache) whose forward block wrote it
      const uint32_t full = grid & ~7u;
      if (bid < full) bid = full - 8u - (bid & ~7u) + (bid & 7u);
    }
    slice = 0;
    O = p.O;
    if (p.O > 1) {  // a 3-D problem: the grid holds the blocks of slice 0, then those of slice 1, ...
      const uint32_t sl = bid / (uint32_t)p.tiles_per_slice;
      bid -= sl * (uint32_t)p.tiles_per_slice;
      slice = sl;
    }
    rt = bid / nct;
    ct = bid - rt * nct;
    // a block covers p.col_chunks consecutive column chunks of TX * VEC columns (1 unless the
    // kernel was compiled to take several per row step); c0 is the lane's column in the first
    const int cc = p.col_chunks > 0 ? p.col_chunks : 1;
    chunk_cols = TX * VEC;
    chunk_bytes = (uint32_t)chunk_cols * (uint32_t)sizeof(T);
    c0 = (((int64_t)ct * cc) << ltx) * VEC + (int64_t)tx * VEC;
    colvalid = c0 < p.C;
    // Which rows a block takes.  Contiguous: steps * TY consecutive rows.  Interleaved: its
    // k-th row step is step k * n_rt + rt of the whole problem, so that the blocks resident at
    // one time sweep one contiguous band of every plane together (a contiguous run per block
    // puts the blocks a large power of two apart, on the same memory channels).
    if (p.interleave) {
      r_first = (int64_t)rt * TY;
      r_step = (int64_t)p.n_rt * TY;
    } else {
      r_first = (int64_t)rt * rows_pb;
      r_step = TY;
    }
    interior = r_first + (p.steps - 1) * r_step + TY <= p.R && (((((int64_t)ct + 1) * cc) << ltx) * VEC) <= p.C;
    // with one row stride common to the full-shape views, one byte offset per lane serves the
    // adjoints, every plane and every full gradient at every row step
    shift = p.ragged && colvalid && c0 + VEC > p.C ? (int)(c0 + VEC - p.C) : 0;
    const int64_t cl = c0 - shift;  // the lane's first load column
    col_off = (uint32_t)cl * (uint32_t)sizeof(T);
    lane_uniform = ((uint32_t)ty * (uint32_t)p.row_stride + (uint32_t)cl) * (uint32_t)sizeof(T);
    lds_row = reinterpret_cast<A *>(smem + p.lds_row_off);
    lds_col = reinterpret_cast<A *>(smem + p.lds_col_off);
    lds_all = reinterpret_cast<A *>(smem + p.lds_all_off);
    for (int s = 0; s < p.n_col_slots; ++s)
#pragma unroll
      for (int v = 0; v < VEC; ++v) lds_col[(s * kBlock + tid) * VEC + v] = AT::zero();
    for (int s = 0; s < p.n_all_slots; ++s) lds_all[s * kBlock + tid] = AT::zero();
  }
  // row of this lane at row step k of the block
  BD_DEV int64_t row(int k) const { return r_first + ty + k * r_step; }
  // Addressing of row step k.  A step that starts past the last row (only lanes outside the
  // problem, which read a view's first vector of the step and discard it) is moved to row 0.
  template <bool US>
  BD_DEV RowStep<T, US> step(const BwdTiledParams &p, int k) const {
    int64_t r0 = r_first + k * r_step;
    r0 = r0 < p.R ? r0 : 0;
    return RowStep<T, US>{r0, slice, (slice * p.outer_stride + r0 * p.row_stride) * (int64_t)sizeof(T), lane_uniform, (uint32_t)ty, col_off};
  }
  // row behind the block-local row index q = k * TY + ty
  BD_DEV int64_t row_of_local(int q) const {
    const int lty = 8 - ltx;  // kBlock = 256 lanes = TY * TX
    return r_first + (q >> lty) * r_step + (q & (TY - 1));
  }
};

// one vector of a plane (`base`: the plane at the row step's first row; `off`: the lane's offset
// from there); lanes outside the problem read offset 0 and get zeros
// RAGGED: the vector may lie at any element boundary, and in an edge block the row's last lane,
// which has loaded `shift` columns to the left of its own, gets its columns moved to the front
template <class T, int VEC, bool EDGE, bool RAGGED = false>
BD_DEV void load_plane(const void *base, uint32_t off, bool valid, T (&x)[VEC], int shift = 0) {
  if (EDGE) {
    load_vec<T, VEC, kBwdLoadNt, RAGGED>(at<const T>(base, valid ? off : 0u), x);
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = valid ? x[v] : T(0);
    if constexpr (RAGGED) unshift<T, VEC>(x, shift);
  } else {
    load_vec<T, VEC, kBwdLoadNt, RAGGED>(at<const T>(base, off), x);
  }
}

// the per-class treatment of one gradient at one row step
// `gbase`: the gradient's own view at the row step's first row; `off`: the lane's byte offset from there
// (RAGGED: `off` is where the lane's loads go, `shift` columns left of its own first column)
// NTS: the gradient is written with the nontemporal hint
template <class T, int VEC, int MAXM, bool EDGE, bool RAGGED = false, bool NTS = false>
BD_DEV void apply_full(const void *gbase, const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC], uint32_t off,
                       bool valid, int shift = 0) {
  T o[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) o[v] = wide_dot<T, MAXM, VEC>(adj, P, v);
  if (!EDGE || valid) {
    if constexpr (RAGGED && EDGE) store_ragged<T, VEC>(at<T>(gbase, off), o, shift);
    else store_vec<T, VEC, RAGGED, NTS>(at<T>(gbase, off), o);
  }
}
// row sums in two halves: a lane's own columns first (over as many column chunks as the kernel
// holds), then once per row step the reduction over the row's lanes and the store
template <class T, int VEC, int MAXM>
BD_DEV void rowsum_lane(typename acc_traits<T>::type &rs, const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC]) {
  using AT = acc_traits<T>;
#pragma unroll
  for (int v = 0; v < VEC; ++v)
#pragma unroll
    for (int i = 0; i < MAXM; ++i) AT::add_prod(rs, adj[i][v], P[i][v]);
}
template <class T, int VEC>
BD_DEV void rowsum_finish(const BwdTiledParams &p, const BwdGeom<T, VEC> &g, const BwdEntry &en,
                          typename acc_traits<T>::type rs, int64_t r, int ri) {
  using AT = acc_traits<T>;
  using A = typename AT::type;
  if (g.ltx >= 6) {  // the wavefront lies inside one row
    rs = wave_total<T, A>(rs);
    if ((g.tid & 63) == 0 && r < p.R) {
      if (g.ltx > 6)
        g.lds_row[(en.slot * g.rows_pb + ri) * g.wpr + (g.tx >> 6)] = rs;
      else if (en.direct)
        static_cast<T *>(en.g.p)[g.slice * en.g.so + r * en.g.sr] = AT::fin(rs);
      else
        reinterpret_cast<A *>(p.ws + en.ws_off)[(r * g.O + g.slice) * p.n_ct + g.ct] = rs;
    }
  } else {  // several rows per wavefront: segmented butterfly
    rs = seg_reduce<T, A>(rs, g.ltx);
    if (g.tx == 0 && r < p.R) {
      if (en.direct)
        static_cast<T *>(en.g.p)[g.slice * en.g.so + r * en.g.sr] = AT::fin(rs);
      else
        reinterpret_cast<A *>(p.ws + en.ws_off)[(r * g.O + g.slice) * p.n_ct + g.ct] = rs;
    }
  }
}
template <class T, int VEC, int MAXM>
BD_DEV void apply_rowsum(const BwdTiledParams &p, const BwdGeom<T, VEC> &g, const BwdEntry &en,
                         const T (&adj)[MAXM][VEC], const T (&P)[MAXM][VEC], int64_t r, int ri) {
  typename acc_traits<T>::type rs = acc_traits<T>::zero();
  rowsum_lane<T, VEC, MAXM>(rs, adj, P);
  rowsum_finish<T, VEC>(p, g, en, rs, r, ri);
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
        const int64_t r = g.row_of_local(q);
        if (r < p.R) {
          A s = g.lds_row[(en.slot * g.rows_pb + q) * g.wpr];
          for (int w = 1; w < g.wpr; ++w) AT::add(s, g.lds_row[(en.slot * g.rows_pb + q) * g.wpr + w]);
          if (en.direct)
            static_cast<T *>(en.g.p)[g.slice * en.g.so + r * en.g.sr] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[(r * g.O + g.slice) * p.n_ct + g.ct] = s;
        }
      }
    } else if (en.cls == kGradColSum) {
      if (g.ty == 0 && g.colvalid) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          if (g.c0 + v >= p.C) break;  // ragged rows: the last lane holds fewer than VEC columns
          A s = g.lds_col[(en.slot * kBlock + g.tx) * VEC + v];
          for (int y = 1; y < g.TY; ++y) AT::add(s, g.lds_col[(en.slot * kBlock + y * g.TX + g.tx) * VEC + v]);
          if (en.direct)
            static_cast<T *>(en.g.p)[g.slice * en.g.so + (g.c0 + v) * en.g.sc] = AT::fin(s);
          else
            reinterpret_cast<A *>(p.ws + en.ws_off)[((int64_t)g.rt * g.O + g.slice) * p.C + g.c0 + v] = s;
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
          static_cast<T *>(en.g.p)[g.slice * en.g.so] = AT::fin(t);
        else
          reinterpret_cast<A *>(p.ws + en.ws_off)[(int64_t)g.bid * g.O + g.slice] = t;
      }
    }
  }
}

}  // namespace bd
