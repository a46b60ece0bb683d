// Recompute-in-reverse kernels: D(b) applied in the reverse pass (the alternative described
// at the end of Sec. 2.2.3 of arXiv 1810.08297).  Nothing is cached between the passes: one
// kernel reads the arguments and the upstream adjoints, evaluates b on dual numbers again,
// forms t_j = sum_i adj_i * dY_i/dX_j in registers and hands it to the same per-class
// treatment (store / row sum / column sum / full sum) as the plane-reading backward kernels.
#pragma once
#include "bwd_device.h"

namespace bd {

template <class T> struct type_tag { using type = T; };

// a launch's arguments are limited to 4 KiB
static_assert(sizeof(BwdTiledParams) + sizeof(RecomputeArgs) <= 4096, "the recompute kernel's two parameter blocks exceed the kernel argument limit");

// PATTERN: 0 = the class of every gradient is read from the table at run time; otherwise 3 bits
// per differentiable argument (class + 1), and if no class sums over rows the block handles one
// row step without a loop.
constexpr bool pattern_sums_rows(uint64_t pattern) {
  for (int jd = 0; jd < 20; ++jd) {
    const int c = (int)((pattern >> (3 * jd)) & 7u);
    if (c == kGradColSum + 1 || c == kGradAllSum + 1) return true;
  }
  return false;
}
// the same op with every array transposed: row vectors become column vectors and back
constexpr uint64_t transpose_pattern(uint64_t pattern) {
  uint64_t q = 0;
  for (int jd = 0; jd < 20; ++jd) {
    uint64_t c = (pattern >> (3 * jd)) & 7u;
    if (c == kGradRowSum + 1) c = kGradColSum + 1;
    else if (c == kGradColSum + 1) c = kGradRowSum + 1;
    q |= c << (3 * jd);
  }
  return q;
}
// How argument j reaches the lanes when the pattern is fixed at compile time: the class of its
// gradient says along which dims it varies.  Control inputs have no gradient; their form, and
// every form under the run-time pattern, is read from the invariance masks.
enum { kFormRuntime = 0, kFormFull, kFormRowVector, kFormColVector, kFormScalar };
template <class Op, uint64_t PATTERN>
constexpr int arg_form(int j) {
  if (PATTERN == 0 || ((Op::NONDIFF >> j) & 1u)) return kFormRuntime;
  const int jd = popc(~Op::NONDIFF & ((1u << j) - 1u));
  const int cls = (int)((PATTERN >> (3 * jd)) & 7u) - 1;
  return cls == kGradFull ? kFormFull : cls == kGradColSum ? kFormRowVector : cls == kGradRowSum ? kFormColVector : kFormScalar;
}
// RAGGED: rows of any length (at least VEC) and at any element boundary, see unshift.
template <class Op, class T, int VEC, uint64_t PATTERN, bool US, bool RAGGED = false>
__global__ __launch_bounds__(kBlock) void bwdr_tiled_kernel(const BwdTiledParams p, const RecomputeArgs ra) {
  constexpr bool LOOP = PATTERN == 0 || pattern_sums_rows(PATTERN);
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  extern __shared__ __align__(16) unsigned char smem[];
  const BwdGeom<T, VEC> g(p, smem);
  const uint32_t col_off = g.colvalid ? g.col_off : 0u;
  uint32_t colinv_again = ra.col_invariant;
  asm volatile("" : "+s"(colinv_again));
  const int n_steps = LOOP ? p.steps : 1;
  for (int n = 0; n < n_steps; ++n) {
    const int k = p.reverse ? n_steps - 1 - n : n;  // last to first with the tiles
    const int ri = k * g.TY + g.ty;
    const int64_t r = g.row(k);
    const bool valid = g.colvalid && r < p.R;
    const RowStep<T, US> rs = g.template step<US>(p, k);
    // lanes outside the problem read the row step's first vector; a view's offset is its own when
    // the views do not share one row stride
    auto voff = [&](int64_t sr) { return valid ? rs.lane(sr) : 0u; };
    const int64_t r_ld = r < p.R ? r : 0;
    // Arguments.  Where the pattern fixes an argument's broadcast form the matching load is
    // issued unconditionally.  Otherwise (control inputs, run-time pattern) both forms go into
    // registers of their own, the one that does not apply skipped by a uniform branch and left
    // as zero bits, and the two are OR-ed together afterwards; a lane's vector stays one value
    // (one register tuple) and passes through an opaque point after the last load, or the
    // compiler consumes single elements inside the conditional blocks and waits there for the
    // load it has just issued.
    using LV = typename lane_vec<T, VEC>::type;
    LV avec[N];
    T asc[N];
    static_for<0, N>([&](auto J) {
      constexpr int j = decltype(J)::value;
      constexpr int form = arg_form<Op, PATTERN>(j);
      avec[j] = LV(T(0));
      if constexpr (form == kFormFull)
        avec[j] = load_lane_vec<T, VEC, kRecArgNt, RAGGED>(at<const T>(rs.base(ra.arg_p[j], ra.arg_sr[j], ra.arg_so[j]), voff(ra.arg_sr[j])));
      else if constexpr (form == kFormRowVector)
        avec[j] = load_lane_vec<T, VEC, kRecArgNt, RAGGED>(at<const T>(static_cast<const T *>(ra.arg_p[j]) + g.slice * ra.arg_so[j], col_off));
      else if constexpr (form == kFormRuntime) {
        const bool colinv = (ra.col_invariant >> j) & 1u;
        if constexpr (PATTERN != 0) {
          // a control input beside unconditional loads: no branch either -- where the vector
          // form does not apply the lane reads the first adjoint's vector instead (valid
          // memory that is loaded anyway) and the result is replaced by zero bits
          const bool rowinv = (ra.row_invariant >> j) & 1u;
          const LV x = load_lane_vec<T, VEC, false, RAGGED>(colinv   ? at<const T>(rs.base(p.adj[0]), voff(p.adj[0].sr))
                                             : rowinv ? at<const T>(static_cast<const T *>(ra.arg_p[j]) + g.slice * ra.arg_so[j], col_off)
                                                      : at<const T>(rs.base(ra.arg_p[j], ra.arg_sr[j], ra.arg_so[j]), voff(ra.arg_sr[j])));
          avec[j] = colinv ? LV(T(0)) : x;
        } else if (!colinv) {
          avec[j] = load_lane_vec<T, VEC, kRecArgNt, RAGGED>(((ra.row_invariant >> j) & 1u) ? at<const T>(static_cast<const T *>(ra.arg_p[j]) + g.slice * ra.arg_so[j], col_off)
                                                                                           : at<const T>(rs.base(ra.arg_p[j], ra.arg_sr[j], ra.arg_so[j]), voff(ra.arg_sr[j])));
        }
      }
    });
    static_for<0, N>([&](auto J) {
      constexpr int j = decltype(J)::value;
      constexpr int form = arg_form<Op, PATTERN>(j);
      asc[j] = T(0);
      if constexpr (form == kFormColVector)
        asc[j] = static_cast<const T *>(ra.arg_p[j])[g.slice * ra.arg_so[j] + r_ld * ra.arg_sr[j]];
      else if constexpr (form == kFormScalar)
        asc[j] = static_cast<const T *>(ra.arg_p[j])[g.slice * ra.arg_so[j]];
      else if constexpr (form == kFormRuntime) {
        const bool colinv = (colinv_again >> j) & 1u;
        if constexpr (PATTERN != 0) {  // element 0 exists for every argument
          const T x = static_cast<const T *>(ra.arg_p[j])[g.slice * ra.arg_so[j] + ((colinv && !((ra.row_invariant >> j) & 1u)) ? r_ld * ra.arg_sr[j] : 0)];
          asc[j] = colinv ? x : T(0);
        } else if (colinv) {
          asc[j] = static_cast<const T *>(ra.arg_p[j])[g.slice * ra.arg_so[j] + (((ra.row_invariant >> j) & 1u) ? 0 : r_ld * ra.arg_sr[j])];
        }
      }
    });
    T adj[M][VEC];
#pragma unroll
    for (int i = 0; i < M; ++i) load_plane<T, VEC, true, RAGGED>(rs.base(p.adj[i]), rs.lane(p.adj[i].sr), valid, adj[i], g.shift);
#pragma unroll
    for (int j = 0; j < N; ++j)  // the opaque point after the last load
      if (arg_form<Op, PATTERN>(j) == kFormRuntime) {
        asm volatile("" : "+v"(asc[j]));
        asm volatile("" : "+v"(avec[j]));
      }
    T a[N][VEC];
    static_for<0, N>([&](auto J) {
      constexpr int j = decltype(J)::value;
      constexpr int form = arg_form<Op, PATTERN>(j);
      T x[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) x[v] = lane_elem<T, VEC>(avec[j], v);
      if constexpr (RAGGED) unshift<T, VEC>(x, g.shift);
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        if constexpr (form == kFormFull || form == kFormRowVector)
          a[j][v] = x[v];
        else if constexpr (form == kFormColVector || form == kFormScalar)
          a[j][v] = asc[j];
        else
          a[j][v] = or_bits(x[v], asc[j]);
      }
    });
    Y y[VEC][M];
#pragma unroll
    for (int v = 0; v < VEC; ++v) (void)eval_op<Op, T, VEC>(a, v, y[v], std::make_index_sequence<N>{});

    static_for<0, ND>([&](auto JD) {
      constexpr int jd = decltype(JD)::value;
      const int e = ra.entry_of[jd];
      if (e >= 0) {
        const BwdEntry &en = p.e[e];
        T P[M][VEC];
#pragma unroll
        for (int i = 0; i < M; ++i)
#pragma unroll
          for (int v = 0; v < VEC; ++v)  // nothing from columns past the row's end: 0 x inf would reach the sums
            P[i][v] = valid && (!RAGGED || v + g.shift < VEC) ? y[v][i].template partial<jd>() : T(0);
        constexpr int fixed = (int)((PATTERN >> (3 * jd)) & 7u);
        const int cls = fixed ? fixed - 1 : en.cls;
        if (cls == kGradFull)
          apply_full<T, VEC, M, true, RAGGED>(rs.base(en.g), adj, P, rs.lane(en.g.sr), valid, g.shift);
        else if (cls == kGradRowSum)
          apply_rowsum<T, VEC, M>(p, g, en, adj, P, r, ri);
        else if (cls == kGradColSum)
          apply_colsum<T, VEC, M>(g, en, adj, P);
        else if (cls == kGradAllSum)
          apply_allsum<T, VEC, M>(g, en, adj, P);
      }
    });
  }
  bwd_finalize<T, VEC>(p, g);
}

// fixed: 0 = the pattern is read at run time, 1 = the call has the op's compiled-in pattern,
// 2 = it has that pattern transposed
template <class Op>
hipError_t launch_bwdr_tiled(int dt, int vec, int fixed, const BwdTiledParams &p, const RecomputeArgs &ra,
                             dim3 grid, size_t lds, const Launch &s) {
  constexpr uint64_t PAT = Op::RECOMPUTE_PATTERN, PAT_T = transpose_pattern(Op::RECOMPUTE_PATTERN);
  auto go = [&](auto type_tag, auto vec_tag, auto us_tag) {
    using T = typename decltype(type_tag)::type;
    constexpr int V = decltype(vec_tag)::value;
    constexpr bool US = decltype(us_tag)::value;
    if constexpr (V * sizeof(T) == 16 && US) {
      if (p.ragged) {  // planned for the widest vector and one common row stride; the compiled-in pattern or the run-time one
        if (fixed == 1) return launch((bwdr_tiled_kernel<Op, T, V, PAT, true, true>), grid, dim3(kBlock), lds, s, p, ra);
        return launch((bwdr_tiled_kernel<Op, T, V, 0ull, true, true>), grid, dim3(kBlock), lds, s, p, ra);
      }
    }
    if constexpr (V * sizeof(T) == 16) {  // the fixed patterns exist for the widest vector only
      if (fixed == 1) return launch((bwdr_tiled_kernel<Op, T, V, PAT, US>), grid, dim3(kBlock), lds, s, p, ra);
      if constexpr (PAT_T != PAT)
        if (fixed == 2) return launch((bwdr_tiled_kernel<Op, T, V, PAT_T, US>), grid, dim3(kBlock), lds, s, p, ra);
    }
    launch((bwdr_tiled_kernel<Op, T, V, 0ull, US>), grid, dim3(kBlock), lds, s, p, ra);
  };
  if (!p.uniform_stride && !Op::STRIDED) return hipErrorNotSupported;  // the host refuses such calls
  if (p.ragged && !(p.uniform_stride && vec * (dt == BCAST_F32 ? 4 : 8) == 16)) return hipErrorInvalidValue;
  auto with_stride = [&](auto type_tag, auto vec_tag) {
    if (p.uniform_stride) go(type_tag, vec_tag, std::true_type{});
    else if constexpr (Op::STRIDED) go(type_tag, vec_tag, std::false_type{});  // views with row strides of their own
  };
  if (dt == BCAST_F32) {
    if (vec == 4) with_stride(type_tag<float>{}, std::integral_constant<int, 4>{});
    else with_stride(type_tag<float>{}, std::integral_constant<int, 1>{});
  } else {
    if (vec == 2) with_stride(type_tag<double>{}, std::integral_constant<int, 2>{});
    else with_stride(type_tag<double>{}, std::integral_constant<int, 1>{});
  }
  return hipGetLastError();
}

}  // namespace bd

#define BD_DEFINE_OP_RECOMPUTE(OPTYPE, IDENT)                                                              \
  hipError_t bd_bwdr_tiled_##IDENT(int dt, int vec, int fixed, const bd::BwdTiledParams &p,                \
                                   const bd::RecomputeArgs &ra, dim3 g, size_t lds, const bd::Launch &s) {       \
    return bd::launch_bwdr_tiled<OPTYPE>(dt, vec, fixed, p, ra, g, lds, s);                                \
  }                                                                                                        \
  uint64_t bd_bwdr_pattern_##IDENT() { return OPTYPE::RECOMPUTE_PATTERN; }
