// Recompute-in-reverse kernels: D(b) applied in the reverse pass (the alternative described
// at the end of Sec. 2.2.3 of arXiv 1810.08297).  Nothing is cached between the passes: one
// kernel reads the arguments and the upstream adjoints, evaluates b on dual numbers again,
// forms t_j = sum_i adj_i * dY_i/dX_j in registers and hands it to the same per-class
// treatment (store / row sum / column sum / full sum) as the plane-reading backward kernels.
#pragma once
#include "bwd_device.h"

namespace bd {

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
template <class Op, class T, int VEC, uint64_t PATTERN>
__global__ __launch_bounds__(kBlock) void bwdr_tiled_kernel(const BwdTiledParams p, const RecomputeArgs ra) {
  constexpr bool LOOP = PATTERN == 0 || pattern_sums_rows(PATTERN);
  constexpr int N = Op::N, M = Op::M;
  constexpr int ND = N - popc(Op::NONDIFF);
  using Y = Dual<T, (ND >= 32 ? 0xffffffffu : ((1u << ND) - 1u))>;
  extern __shared__ __align__(16) unsigned char smem[];
  const BwdGeom<T, VEC> g(p, smem);
  const bool nt = p.nt_store != 0;
  const uint32_t col_off = g.colvalid ? (uint32_t)g.c0 * (uint32_t)sizeof(T) : 0u;
  uint32_t colinv_again = ra.col_invariant;
  asm volatile("" : "+s"(colinv_again));
  uint32_t off = g.off0;
  for (int k = 0; k < (LOOP ? p.steps : 1); ++k, off += g.off_step) {
    const int ri = k * g.TY + g.ty;
    const int64_t r = g.row(k);
    const bool valid = g.colvalid && r < p.R;
    const uint32_t off_ld = valid ? off : 0u;       // lanes outside the problem read element 0
    const int64_t r_ld = r < p.R ? r : 0;
    // arguments: both forms into registers of their own, all loads in flight together
    T avec[N][VEC], asc[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) avec[j][v] = T(0);
      if (!((ra.col_invariant >> j) & 1u))
        load_vec<T, VEC, BD_REC_ARG_NT != 0>(at<const T>(ra.arg_p[j], ((ra.row_invariant >> j) & 1u) ? col_off : off_ld), avec[j]);
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      asc[j] = T(0);
      if ((colinv_again >> j) & 1u)
        asc[j] = static_cast<const T *>(ra.arg_p[j])[((ra.row_invariant >> j) & 1u) ? 0 : r_ld * ra.arg_sr[j]];
    }
    T adj[M][VEC];
#pragma unroll
    for (int i = 0; i < M; ++i) load_plane<T, VEC, true>(p.adj[i].p, off, valid, adj[i]);
    T a[N][VEC];
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
      for (int v = 0; v < VEC; ++v) a[j][v] = or_bits(avec[j][v], asc[j]);
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
          for (int v = 0; v < VEC; ++v) P[i][v] = valid ? y[v][i].template partial<jd>() : T(0);
        constexpr int fixed = (int)((PATTERN >> (3 * jd)) & 7u);
        const int cls = fixed ? fixed - 1 : en.cls;
        if (cls == kGradFull)
          apply_full<T, VEC, M, true>(en, adj, P, off, valid, nt);
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

template <class Op>
hipError_t launch_bwdr_tiled(int dt, int vec, bool fixed_pattern, const BwdTiledParams &p, const RecomputeArgs &ra,
                             dim3 grid, size_t lds, hipStream_t s) {
#define BD_GO(T, V, PAT) launch((bwdr_tiled_kernel<Op, T, V, PAT>), grid, dim3(kBlock), lds, s, p, ra)
  if (dt == BCAST_F32) {
    if (vec == 4) {
      if (fixed_pattern) BD_GO(float, 4, Op::RECOMPUTE_PATTERN); else BD_GO(float, 4, 0ull);
    } else {
      BD_GO(float, 1, 0ull);
    }
  } else {
    if (vec == 2) {
      if (fixed_pattern) BD_GO(double, 2, Op::RECOMPUTE_PATTERN); else BD_GO(double, 2, 0ull);
    } else {
      BD_GO(double, 1, 0ull);
    }
  }
#undef BD_GO
  return hipGetLastError();
}

}  // namespace bd

#define BD_DEFINE_OP_RECOMPUTE(OPTYPE, IDENT)                                                              \
  hipError_t bd_bwdr_tiled_##IDENT(int dt, int vec, bool fixed, const bd::BwdTiledParams &p,               \
                                   const bd::RecomputeArgs &ra, dim3 g, size_t lds, hipStream_t s) {       \
    return bd::launch_bwdr_tiled<OPTYPE>(dt, vec, fixed, p, ra, g, lds, s);                                \
  }                                                                                                        \
  uint64_t bd_bwdr_pattern_##IDENT() { return OPTYPE::RECOMPUTE_PATTERN; }
