// Dual-number forward kernels: one launch evaluates b on x_j + eps_j for every element and
// writes the M values and the M x N_d partial planes (Sec. 2.2.2; fused primal + tangent
// evaluation, Sec. 2.2.3).  HBM-bound: no matrix cores; the work is laid out so that every
// wavefront memory instruction moves 64 x 16 contiguous bytes per plane.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kparams.h"
#include "launch.h"
#include "ops.h"

namespace bd {

// `type`: a lane's vector, aligned to its size.  `unaligned`: the same vector at any element
// boundary, for rows whose length or start is not a multiple of the vector (global memory
// takes multi-dword accesses at dword boundaries; they are only slower across cache lines).
template <class T, int VEC> struct vec_of;
template <> struct vec_of<float, 4> {
  typedef float type __attribute__((ext_vector_type(4)));
  typedef float unaligned __attribute__((ext_vector_type(4), aligned(4)));
};
template <> struct vec_of<float, 2> {
  typedef float type __attribute__((ext_vector_type(2)));
  typedef float unaligned __attribute__((ext_vector_type(2), aligned(4)));
};
template <> struct vec_of<double, 2> {
  typedef double type __attribute__((ext_vector_type(2)));
  typedef double unaligned __attribute__((ext_vector_type(2), aligned(8)));
};

// Cache policy of the streaming loads.  Arguments, adjoints and planes are read once per
// launch, so their loads carry the nontemporal hint: measured on MI355X the backward kernel
// drops from 101 to 78 us on the HM-LSTM workload (lines that will not be reused no longer
// displace the freshly written planes from the memory-side cache).  The recompute kernels read
// the arguments the values-only forward launch has just read, and load them plainly.
constexpr bool kFwdArgNt = true;   // arguments of the plane-writing forward kernel
constexpr bool kBwdLoadNt = true;  // adjoints and planes in the backward kernels
constexpr bool kRecArgNt = false;  // arguments in the recompute kernels

template <class T, int VEC, bool NT = false, bool UNALIGNED = false>
BD_DEV void load_vec(const T *p, T (&x)[VEC]) {
  if constexpr (VEC == 1) {
    x[0] = NT ? __builtin_nontemporal_load(p) : *p;
  } else {
    using V = std::conditional_t<UNALIGNED, typename vec_of<T, VEC>::unaligned, typename vec_of<T, VEC>::type>;
    typename vec_of<T, VEC>::type v = NT ? __builtin_nontemporal_load(reinterpret_cast<const V *>(p)) : *reinterpret_cast<const V *>(p);
#pragma unroll
    for (int k = 0; k < VEC; ++k) x[k] = v[k];
  }
}
// A lane's VEC consecutive elements held as ONE value (a register tuple), for code that must
// keep a conditionally loaded vector whole until all loads have been issued.
template <class T, int VEC> struct lane_vec { using type = typename vec_of<T, VEC>::type; };
template <class T> struct lane_vec<T, 1> { using type = T; };
template <class T, int VEC> struct lane_vec_unaligned { using type = typename vec_of<T, VEC>::unaligned; };
template <class T> struct lane_vec_unaligned<T, 1> { using type = T; };
template <class T, int VEC, bool NT = false, bool UNALIGNED = false>
BD_DEV typename lane_vec<T, VEC>::type load_lane_vec(const T *p) {
  using V = std::conditional_t<UNALIGNED, typename lane_vec_unaligned<T, VEC>::type, typename lane_vec<T, VEC>::type>;
  return NT ? __builtin_nontemporal_load(reinterpret_cast<const V *>(p)) : *reinterpret_cast<const V *>(p);
}
template <class T, int VEC>
BD_DEV T lane_elem(const typename lane_vec<T, VEC>::type &x, int k) {
  if constexpr (VEC == 1) return x; else return x[k];
}

// NTS: with the nontemporal hint, fixed at compile time.  (A run-time choice written as a plain
// if / else does not survive: the compiler merges the two stores, which differ in nothing but the
// hint, into one without it.  store_at below is the form that does.)
template <class T, int VEC, bool UNALIGNED = false, bool NTS = false>
BD_DEV void store_vec(T *p, const T (&x)[VEC]) {
  if constexpr (VEC == 1) {
    if constexpr (NTS) __builtin_nontemporal_store(x[0], p); else *p = x[0];
  } else {
    using V = std::conditional_t<UNALIGNED, typename vec_of<T, VEC>::unaligned, typename vec_of<T, VEC>::type>;
    typename vec_of<T, VEC>::type v;
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = x[k];
    if constexpr (NTS) __builtin_nontemporal_store(v, reinterpret_cast<V *>(p)); else *reinterpret_cast<V *>(p) = v;
  }
}

// Rows whose length is not a multiple of the vector (RAGGED kernels).  The lane that holds a
// row's last, partial vector -- columns c0 .. C-1, fewer than VEC -- loads the vector that ENDS
// with the row instead, `shift` = c0 + VEC - C columns to the left: always whole, always inside
// the row (C >= VEC).  unshift moves the lane's own columns to the front and clears the rest, so
// that element v is column c0 + v everywhere, zero past the row's end.
template <class T, int VEC>
BD_DEV void unshift(T (&x)[VEC], int shift) {
  if constexpr (VEC > 1) {
    T y[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      y[v] = T(0);
#pragma unroll
      for (int s = 0; s + v < VEC; ++s) y[v] = shift == s ? x[v + s] : y[v];
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = y[v];
  }
}
// `p`: where the lane's loads go (its first column less `shift`).  A whole vector is stored as
// one; the row's last lane stores its VEC - shift columns one by one.
template <class T, int VEC>
BD_DEV void store_ragged(T *p, const T (&x)[VEC], int shift) {
  if (shift == 0) {
    store_vec<T, VEC, true>(p, x);
  } else {
#pragma unroll
    for (int v = 0; v < VEC; ++v)
      if (v + shift < VEC) p[shift + v] = x[v];
  }
}

// base + byte offset; with a uniform base and a 32-bit lane offset this is the
// scalar-base + vector-offset addressing mode: no per-plane address arithmetic
// Kernel arguments are read with scalar loads, and the compiler issues each where it is first
// needed: behind uniform branches that means one load, one wait, one use, again and again -- some
// thirty round trips to the scalar cache in a block that lives a few microseconds.  Folding the
// values a block will need into one word and handing that word to an empty asm makes all their
// loads issue together and complete at that point; the values themselves stay what they were
// (pointers keep their address space, so accesses keep the scalar-base form).
BD_DEV uint32_t low_word(const void *x) { return (uint32_t)reinterpret_cast<uintptr_t>(x); }
BD_DEV uint32_t low_word(int64_t x) { return (uint32_t)x; }
BD_DEV uint32_t low_word(int32_t x) { return (uint32_t)x; }
BD_DEV uint32_t low_word(uint32_t x) { return x; }
BD_DEV void arrived(uint32_t folded) { asm volatile("" ::"s"(folded)); }

template <class T>
BD_DEV T *at(const void *base, uint32_t byte_off) {
  // The empty asm pins the zero-extension of the offset to the basic block of the access;
  // instruction selection only folds base + zext(offset) into one instruction when it sees
  // both there (accesses sit behind uniform null-pointer and bounds branches).
  asm("" : "+v"(byte_off));
  return reinterpret_cast<T *>(const_cast<char *>(static_cast<const char *>(base)) + byte_off);
}

// One vector to base + byte offset, with or without the nontemporal hint, chosen at run time by a
// value that is the same for the whole block.  The two empty asm statements keep the two stores
// from being merged into one without the hint, and forming the address inside each branch keeps
// the scalar-base + lane-offset form for both.  (In a kernel that loops over row steps the branch
// costs: the backward kernels take the hint as a template parameter instead.)
template <class T, int VEC, bool UNALIGNED = false>
BD_DEV void store_at(const void *base, uint32_t byte_off, const T (&x)[VEC], bool nt) {
  using V = std::conditional_t<VEC == 1, T, std::conditional_t<UNALIGNED, typename lane_vec_unaligned<T, VEC>::type, typename lane_vec<T, VEC>::type>>;
  typename lane_vec<T, VEC>::type v;
  if constexpr (VEC == 1) {
    v = x[0];
  } else {
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] = x[k];
  }
  if (nt) {
    asm volatile("" ::: "memory");
    __builtin_nontemporal_store(v, reinterpret_cast<V *>(at<T>(base, byte_off)));
    asm volatile("" ::: "memory");
  } else {
    *reinterpret_cast<V *>(at<T>(base, byte_off)) = v;
  }
}

// Where the lanes of one row step find their vectors in a view whose rows are `sr` elements
// apart: a 64-bit part that is the same for the whole block (the view's base moved to the
// step's first row; scalar registers) and a 32-bit part of the lane's own (its row within the
// step and its column).  Views of any size can be addressed this way; the host only has to see
// that one row step of a view, TY rows, spans less than 4 GiB.  With one row stride common to
// all full-shape views (US) both parts are computed once and serve every such view.
template <class T, bool US>
struct RowStep {
  int64_t row0;           // first row of the step (within the block's slice)
  int64_t slice;          // the block's index along the outer dim of a 3-D problem (0 otherwise)
  int64_t uniform_bytes;  // US: (slice * the common outer stride + row0 * the common row stride) * sizeof(T)
  uint32_t lane_uniform;  // US: (lane's row in the step * the common row stride + lane's column) * sizeof(T)
  uint32_t ty, col_off;   // lane's row in the step; lane's column * sizeof(T)
  // a view that varies along rows and columns: its rows `sr`, its slices `so` elements apart
  BD_DEV const void *base(const void *p, int64_t sr, int64_t so) const {
    return static_cast<const char *>(p) + (US ? uniform_bytes : (slice * so + row0 * sr) * (int64_t)sizeof(T));
  }
  BD_DEV const void *base(const TView &v) const { return base(v.p, v.sr, v.so); }
  BD_DEV const void *base(const SView &v) const { return base(v.p, v.sr, v.so); }
  BD_DEV uint32_t lane(int64_t sr) const {
    return US ? lane_uniform : ty * (uint32_t)sr * (uint32_t)sizeof(T) + col_off;
  }
};

BD_DEV float or_bits(float a, float b) { return __uint_as_float(__float_as_uint(a) | __float_as_uint(b)); }
BD_DEV double or_bits(double a, double b) {
  return __longlong_as_double(__double_as_longlong(a) | __double_as_longlong(b));
}

template <class Op, class T, int J, bool SEEDED = true>
BD_DEV auto make_arg(T x) {
  if constexpr ((Op::NONDIFF >> J) & 1u)
    return x;  // control input: a plain scalar, no perturbation
  else if constexpr (SEEDED)
    return seed<T, popc(~Op::NONDIFF & ((1u << J) - 1u))>(x);
  else
    return Dual<T, 0u>(x);  // values only: a dual that depends on no perturbation
}
template <class Op, class T, int VEC, class Y, size_t... J>
BD_DEV int eval_op(const T (&a)[Op::N][VEC], int v, Y *y, std::index_sequence<J...>) {
  return Op::apply(y, make_arg<Op, T, (int)J, (Y::mask != 0u)>(a[J][v])...);
}

// Tiled kernel for problems of two merged dims, or of three (a batch of 2-D slices: see TView).
// Block = 256 lanes arranged TY x TX over TY rows of one slice; a lane owns VEC
// consecutive columns of one row.  Stride-0 arguments are served from registers: a column
// vector or scalar is one broadcast load per lane, a row vector one vector load from its
// only row.  There is deliberately no row loop: with ~30 plane pointers live across a loop
// the scalar register file overflows, and one short-lived block per row tile measured as
// fast as longer-lived ones.
// PARTIALS = false is the values-only launch (no plane requested): the op runs on duals
// without perturbations, so no derivative is computed, and the arguments are loaded with
// plain loads (a recompute backward pass reads them again soon).
// RAGGED: rows of any length (at least VEC) and at any element boundary, see unshift.
template <class Op, class T, int VEC, bool PARTIALS, bool US, bool RAGGED = false>
__global__ __launch_bounds__(kBlock) void fwd_tiled_kernel(const FwdTiledParams p) {
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (!PARTIALS ? 0u : ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  constexpr bool ARG_NT = PARTIALS && kFwdArgNt;
  constexpr bool ROW_VECTORS_APART = ARG_NT;  // the streaming hint is not for row vectors, see below
  // Up front, together: the geometry, the argument pointers and (for arguments read as one value per
  // row) their row strides.  Ops with more arguments than scalar registers allow keep the lazy reads.
  constexpr bool TOGETHER = N + M + (PARTIALS ? M * ND : 0) <= 36;
  const void *ap[N];
#pragma unroll
  for (int j = 0; j < N; ++j) ap[j] = p.arg_p[j];
  if constexpr (TOGETHER) {
    uint32_t f = low_word(p.R) ^ low_word(p.C) ^ low_word(p.log2_tx) ^ p.nt_tiles ^ low_word(p.xcd_remap) ^ low_word(p.n_ct) ^
                 low_word(p.row_stride) ^ low_word(p.O) ^ low_word(p.tiles_per_slice) ^ low_word(p.outer_stride) ^ p.row_invariant ^
                 p.col_invariant;
#pragma unroll
    for (int j = 0; j < N; ++j) f ^= low_word(ap[j]) ^ low_word(p.arg_sr[j]);
    arrived(f);
  }
  const int ltx = p.log2_tx;
  const int tx = threadIdx.x & ((1 << ltx) - 1);
  const int ty = threadIdx.x >> ltx;
  const int TY = kBlock >> ltx;
  const uint32_t nct = (uint32_t)p.n_ct;
  uint32_t bid = blockIdx.x;
  if (p.xcd_remap) bid = (bid & 7u) * (gridDim.x >> 3) + (bid >> 3);  // the host sets this only for grids of 8 n blocks
  const uint32_t walk = bid;  // the tile's place in the order in which the launch writes
  uint32_t slice32 = 0;
  if (p.O > 1) {  // a 3-D problem: the grid holds the blocks of slice 0, then those of slice 1, ...
    slice32 = bid / (uint32_t)p.tiles_per_slice;
    bid -= slice32 * (uint32_t)p.tiles_per_slice;
  }
  const int64_t slice = slice32;
  const uint32_t rt = bid / nct, ct = bid - rt * nct;
  const int64_t c0 = ((((int64_t)ct) << ltx) + tx) * VEC;
  if (c0 >= p.C) return;
  const int64_t r0 = (int64_t)rt * TY;  // the block's first row, the same for all its lanes
  const int64_t r = r0 + ty;
  if (r >= p.R) return;
  // blocks write with the nontemporal hint up to tile nt_tiles of the walk and plainly from there on:
  // what the launch writes last is what a reverse pass reads first and may still find cached
  const bool nt = walk < p.nt_tiles;
  // the row's last lane reads the vector that ends with the row (the host sees that C >= VEC)
  const bool last_tile = ct + 1 == nct;  // uniform: only these blocks hold a row's end
  const int shift = RAGGED && c0 + VEC > p.C ? (int)(c0 + VEC - p.C) : 0;
  const int64_t cl = c0 - shift;
  const uint32_t col_off = (uint32_t)cl * (uint32_t)sizeof(T);
  int64_t aoff[N];  // where the block's slice starts in each argument, in elements
#pragma unroll
  for (int j = 0; j < N; ++j) aoff[j] = 0;
  if (p.O > 1) {
#pragma unroll
    for (int j = 0; j < N; ++j) aoff[j] = slice * p.arg_so[j];
  }
  const RowStep<T, US> rs{r0, slice, (slice * p.outer_stride + r0 * p.row_stride) * (int64_t)sizeof(T),
                          ((uint32_t)ty * (uint32_t)p.row_stride + (uint32_t)cl) * (uint32_t)sizeof(T), (uint32_t)ty, col_off};

  // Every argument is fetched in whichever of two forms applies -- a vector for arguments
  // that vary along the columns, one broadcast element otherwise -- into registers of its
  // own; the form that does not apply is skipped by a uniform branch and reads as zero
  // bits, and the two are OR-ed together afterwards.  Keeping the forms apart (the second
  // test goes through a copy of the mask the compiler cannot see through, or it would fold
  // the two forms into one register again) lets all loads be in flight together instead of
  // each waiting for the one before.
  uint32_t colinv_again = p.col_invariant;
  asm volatile("" : "+s"(colinv_again));
  T avec[N][VEC], asc[N];
#pragma unroll
  for (int j = 0; j < N; ++j) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) avec[j][v] = T(0);
    if constexpr (ROW_VECTORS_APART) {
      if (!(((p.col_invariant | p.row_invariant) >> j) & 1u))  // from this row
        load_vec<T, VEC, ARG_NT, RAGGED>(at<const T>(rs.base(ap[j], p.arg_sr[j], p.arg_so[j]), rs.lane(p.arg_sr[j])), avec[j]);
    } else {
      if (!((p.col_invariant >> j) & 1u))  // from this row, or (row vectors) from the only row
        load_vec<T, VEC, ARG_NT, RAGGED>(((p.row_invariant >> j) & 1u) ? at<const T>(static_cast<const T *>(ap[j]) + aoff[j], col_off)
                                                                         : at<const T>(rs.base(ap[j], p.arg_sr[j], p.arg_so[j]), rs.lane(p.arg_sr[j])), avec[j]);
    }
  }
  // Row vectors, in the kernels that stream their arguments, are a third form with registers of
  // its own: loaded plainly, behind a test of its own copy of the mask, merged with the others
  // after all loads.  Every row of blocks reads them again and they have to stay in the caches:
  // with the hint their few lines were fetched from memory over and over (the HM-LSTM update with
  // z of shape [1 x C], 8192 x 5120: 1097 us, about 900 us now).  The hint is part of the instruction;
  // choosing it per argument in one set of registers put a branch between every two loads
  // (config 1's forward kernel: 73 instead of 63 us), and loading everything plainly in calls with a
  // row vector cost config 3, which has one, 5 %.
  T arow[ROW_VECTORS_APART ? N : 1][VEC];
  if constexpr (ROW_VECTORS_APART) {
    uint32_t rowvec = p.row_invariant & ~p.col_invariant;
    asm volatile("" : "+s"(rowvec));
#pragma unroll
    for (int j = 0; j < N; ++j) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) arow[j][v] = T(0);
      if ((rowvec >> j) & 1u) load_vec<T, VEC, false, RAGGED>(at<const T>(static_cast<const T *>(ap[j]) + aoff[j], col_off), arow[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < N; ++j) {
    asc[j] = T(0);
    if ((colinv_again >> j) & 1u)  // one value for the row (column vectors) or for everything (scalars)
      asc[j] = static_cast<const T *>(ap[j])[aoff[j] + (((p.row_invariant >> j) & 1u) ? 0 : r * p.arg_sr[j])];
  }
  // the pointers of everything the block writes, fetched together while its loads are in flight
  void *op_[M];
  void *pp[PARTIALS ? M * ND : 1];
#pragma unroll
  for (int i = 0; i < M; ++i) op_[i] = p.out_p[i];
  if constexpr (PARTIALS) {
#pragma unroll
    for (int k = 0; k < M * ND; ++k) pp[k] = p.part_p[k];
  }
  if constexpr (TOGETHER) {
    uint32_t f = low_word(p.branch_p);
#pragma unroll
    for (int i = 0; i < M; ++i) f ^= low_word(op_[i]);
    if constexpr (PARTIALS) {
#pragma unroll
      for (int k = 0; k < M * ND; ++k) f ^= low_word(pp[k]);
    }
    arrived(f);
  }
  // the merge below must not sink into the conditional loads above (each load would then be
  // waited for on its own): the broadcast values pass through an opaque point after all loads
#pragma unroll
  for (int j = 0; j < N; ++j) asm volatile("" : "+v"(asc[j]));
  T a[N][VEC];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    if constexpr (ROW_VECTORS_APART)
#pragma unroll
      for (int v = 0; v < VEC; ++v) avec[j][v] = or_bits(avec[j][v], arow[j][v]);
    if constexpr (RAGGED)
      if (last_tile) unshift<T, VEC>(avec[j], shift);
#pragma unroll
    for (int v = 0; v < VEC; ++v) a[j][v] = or_bits(avec[j][v], asc[j]);
  }
  // stores: whole vectors, or (RAGGED, in the blocks that hold a row's end) the row's last columns one by one
  auto put = [&](const void *base, uint32_t off, const T (&o)[VEC]) {
    if (RAGGED && last_tile) store_ragged<T, VEC>(at<T>(base, off), o, shift);
    else store_at<T, VEC, RAGGED>(base, off, o, nt);
  };
  {
    Y y[VEC][M];
    int br[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) br[v] = eval_op<Op, T, VEC>(a, v, y[v], std::make_index_sequence<N>{});

    T o[VEC];
#pragma unroll
    for (int i = 0; i < M; ++i) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) o[v] = y[v][i].v;
      put(rs.base(op_[i], p.out_sr[i], p.out_so[i]), rs.lane(p.out_sr[i]), o);
    }
    if constexpr (PARTIALS) {
#pragma unroll
      for (int i = 0; i < M; ++i) {
        static_for<0, ND>([&](auto JD) {
          constexpr int jd = decltype(JD)::value;
          void *pl = pp[i * ND + jd];
          if (pl != nullptr) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) o[v] = y[v][i].template partial<jd>();
            put(rs.base(pl, p.part_sr[i * ND + jd], p.part_so[i * ND + jd]), rs.lane(p.part_sr[i * ND + jd]), o);
          }
        });
      }
    }
    if (p.branch_p != nullptr) {
      uint8_t *bp = p.branch_p + slice * p.branch_so + r * p.branch_sr + c0 * p.branch_sc;
      if (RAGGED && last_tile) {
#pragma unroll
        for (int v = 0; v < VEC; ++v)
          if (v + shift < VEC) bp[v * p.branch_sc] = (uint8_t)br[v];
      } else if (VEC == 4 && p.branch_sc == 1 && (reinterpret_cast<uintptr_t>(bp) & 3u) == 0) {  // four ids in one store
        uint32_t w = 0;
#pragma unroll
        for (int v = 0; v < VEC; ++v) w |= (uint32_t)(br[v] & 0xff) << (8 * v);
        *reinterpret_cast<uint32_t *>(bp) = w;
      } else {
#pragma unroll
        for (int v = 0; v < VEC; ++v) bp[v * p.branch_sc] = (uint8_t)br[v];
      }
    }
  }
}

// Linear index -> multi-index over the dims d < nd for which take(d) holds, innermost first.
// 64-bit division is emulated with some hundred instructions; a count below 2^32 (checked on
// the uniform bound `count`) takes the 32-bit form instead.
template <class Take>
BD_DEV void decompose(int64_t linear, int64_t count, int nd, const int64_t *shape, int64_t *idx, Take take) {
  if (count <= 0xffffffffLL) {
    uint32_t rem = (uint32_t)linear;
#pragma unroll
    for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
      if (d < nd && take(d)) {
        const uint32_t s = (uint32_t)shape[d], q = rem / s;
        idx[d] = rem - q * s;
        rem = q;
      }
  } else {
    int64_t rem = linear;
#pragma unroll
    for (int d = BCAST_MAX_DIMS - 1; d >= 0; --d)
      if (d < nd && take(d)) {
        idx[d] = rem % shape[d];
        rem /= shape[d];
      }
  }
}

// Generic kernel: any rank up to BCAST_MAX_DIMS, any strides.  A lane takes VEC consecutive
// elements of the innermost dim: one element in general, a 16-byte vector where the host found
// that every view is contiguous (or constant) along that dim and aligned for it.
template <class Op, class T, int VEC>
__global__ __launch_bounds__(kBlock) void fwd_generic_kernel(const FwdGenericParams p) {
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  const int64_t lane = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (lane >= p.E / VEC) return;
  int64_t idx[BCAST_MAX_DIMS] = {0, 0, 0, 0};
  decompose(lane * VEC, p.E, p.nd, p.shape, idx, [](int) { return true; });
  const int inner = p.nd - 1;
  auto off = [&](const GView &g) {
    int64_t o = 0;
#pragma unroll
    for (int d = 0; d < BCAST_MAX_DIMS; ++d) o += idx[d] * g.s[d];
    return o;
  };
  T a[N][VEC];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const T *src = static_cast<const T *>(p.arg[j].p) + off(p.arg[j]);
    if (VEC > 1 && p.arg[j].s[inner] != 0) {
      load_vec<T, VEC, false>(src, a[j]);
    } else {  // one element per lane, or an argument that is constant along the innermost dim
      const T x = *src;
#pragma unroll
      for (int v = 0; v < VEC; ++v) a[j][v] = x;
    }
  }
  Y y[VEC][M];
  int br[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) br[v] = eval_op<Op, T, VEC>(a, v, y[v], std::make_index_sequence<N>{});
  T o[VEC];
#pragma unroll
  for (int i = 0; i < M; ++i) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) o[v] = y[v][i].v;
    store_vec<T, VEC>(static_cast<T *>(p.out[i].p) + off(p.out[i]), o);
    static_for<0, ND>([&](auto JD) {
      constexpr int jd = decltype(JD)::value;
      const GView &pl = p.part[i * ND + jd];
      if (pl.p != nullptr) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = y[v][i].template partial<jd>();
        store_vec<T, VEC>(static_cast<T *>(pl.p) + off(pl), o);
      }
    });
  }
  if (p.branch.p != nullptr) {
    uint8_t *bp = static_cast<uint8_t *>(p.branch.p) + off(p.branch);
    const int64_t bs = VEC > 1 ? p.branch.s[inner] : 0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) bp[v * bs] = (uint8_t)br[v];
  }
}

// ---- launch wrappers, one pair per op ------------------------------------------------------
template <class T> struct fwd_type { using type = T; };
template <class Op, bool PARTIALS, bool US>
void launch_fwd_tiled_as(int dt, int vec, const FwdTiledParams &p, dim3 grid, const Launch &s) {
  const size_t lds = (size_t)p.lds_bytes;
  auto go = [&](auto type_tag, auto vec_tag, auto ragged_tag) {
    using T = typename decltype(type_tag)::type;
    constexpr int V = decltype(vec_tag)::value;
    constexpr bool RG = decltype(ragged_tag)::value;
    launch((fwd_tiled_kernel<Op, T, V, PARTIALS, US, RG>), grid, dim3(kBlock), lds, s, p);
  };
  using std::integral_constant;
  if constexpr (US) {
    if (p.ragged) {  // planned for the widest vector and one common row stride only
      if (dt == BCAST_F32) go(fwd_type<float>{}, integral_constant<int, 4>{}, std::true_type{});
      else go(fwd_type<double>{}, integral_constant<int, 2>{}, std::true_type{});
      return;
    }
  }
  if (dt == BCAST_F32) {
    if (vec == 4) go(fwd_type<float>{}, integral_constant<int, 4>{}, std::false_type{});
    else if (vec == 2 && US) go(fwd_type<float>{}, integral_constant<int, US ? 2 : 1>{}, std::false_type{});  // views with strides of their own: the widest vector or single elements
    else go(fwd_type<float>{}, integral_constant<int, 1>{}, std::false_type{});
  } else {
    if (vec > 1) go(fwd_type<double>{}, integral_constant<int, 2>{}, std::false_type{});
    else go(fwd_type<double>{}, integral_constant<int, 1>{}, std::false_type{});
  }
}
// vec: what the host planned (for views with strides of their own: the widest vector or 1)
template <class Op>
hipError_t launch_fwd_tiled(int dt, int vec, const FwdTiledParams &p, dim3 grid, const Launch &s) {
  if (p.uniform_stride) {
    if (p.has_partials)
      launch_fwd_tiled_as<Op, true, true>(dt, vec, p, grid, s);
    else
      launch_fwd_tiled_as<Op, false, true>(dt, vec, p, grid, s);
  } else if constexpr (Op::STRIDED) {
    if (p.has_partials)
      launch_fwd_tiled_as<Op, true, false>(dt, vec, p, grid, s);
    else
      launch_fwd_tiled_as<Op, false, false>(dt, vec, p, grid, s);
  } else {
    return hipErrorNotSupported;  // the host sends such ops to the generic kernels
  }
  return hipGetLastError();
}
template <class Op>
hipError_t launch_fwd_generic(int dt, const FwdGenericParams &p, dim3 grid, const Launch &s) {
  // the vector form exists for the ops that are built in every variant (the host asks for it only then)
  if constexpr (Op::STRIDED) {
    if (p.vec > 1) {
      if (dt == BCAST_F32)
        launch((fwd_generic_kernel<Op, float, 4>), grid, dim3(kBlock), 0, s, p);
      else
        launch((fwd_generic_kernel<Op, double, 2>), grid, dim3(kBlock), 0, s, p);
      return hipGetLastError();
    }
  }
  if (p.vec > 1) return hipErrorNotSupported;
  if (dt == BCAST_F32)
    launch((fwd_generic_kernel<Op, float, 1>), grid, dim3(kBlock), 0, s, p);
  else
    launch((fwd_generic_kernel<Op, double, 1>), grid, dim3(kBlock), 0, s, p);
  return hipGetLastError();
}

}  // namespace bd

// Defines the two extern launch functions of one op in the translation unit that uses it.
#define BD_DEFINE_OP(OPTYPE, IDENT)                                                                  \
  hipError_t bd_fwd_tiled_##IDENT(int dt, int vec, const bd::FwdTiledParams &p, dim3 g, const bd::Launch &s) { \
    return bd::launch_fwd_tiled<OPTYPE>(dt, vec, p, g, s);                                           \
  }                                                                                                  \
  hipError_t bd_fwd_generic_##IDENT(int dt, const bd::FwdGenericParams &p, dim3 g, const bd::Launch &s) {  \
    return bd::launch_fwd_generic<OPTYPE>(dt, p, g, s);                                              \
  }
