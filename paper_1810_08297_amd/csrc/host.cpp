// Host side of the library: the op table, argument validation, the broadcast plan
// (shape unification, stride-0 expansion, dim merging -- Sec. 2.1.1 of arXiv 1810.08297:
// size-1 dims are virtually copied and arguments are indexed directly, never materialised),
// launch geometry, and the extern "C" entry points.  Nothing here touches device memory;
// everything is validated before the first launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <atomic>
#include <cstdio>
#include <cstring>
#include <vector>

#include "bcast_dual.h"
#include "kparams.h"
#include "launch_types.h"

using namespace bd;

// ---- launchers defined in the kernel translation units ----------------------------------
#define BD_DECLARE_OP(IDENT)                                                                        \
  hipError_t bd_fwd_tiled_##IDENT(int, int, const FwdTiledParams &, dim3, const Launch &);             \
  hipError_t bd_fwd_generic_##IDENT(int, const FwdGenericParams &, dim3, const Launch &);
#define BD_DECLARE_RECOMPUTE(IDENT)                                                                            \
  hipError_t bd_bwdr_tiled_##IDENT(int, int, int, const BwdTiledParams &, const RecomputeArgs &, dim3, size_t,  \
                                   const Launch &);                                                               \
  uint64_t bd_bwdr_pattern_##IDENT();
#define BD_ARITY_LIST(X) \
  X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17) X(18)
BD_DECLARE_OP(hmlstm_update)
BD_DECLARE_OP(update_c)
BD_DECLARE_OP(tanh_xy_b)
BD_DECLARE_OP(branchy5)
BD_DECLARE_OP(cos_x)
BD_DECLARE_OP(scale_xt)
BD_DECLARE_OP(pair3)
BD_DECLARE_OP(linear12)
BD_DECLARE_OP(elementary4)
BD_DECLARE_RECOMPUTE(hmlstm_update)
BD_DECLARE_RECOMPUTE(update_c)
BD_DECLARE_RECOMPUTE(tanh_xy_b)
BD_DECLARE_RECOMPUTE(branchy5)
BD_DECLARE_RECOMPUTE(cos_x)
BD_DECLARE_RECOMPUTE(scale_xt)
BD_DECLARE_RECOMPUTE(pair3)
BD_DECLARE_RECOMPUTE(linear12)
BD_DECLARE_RECOMPUTE(elementary4)
#define BD_DECL_ARITY(K) BD_DECLARE_OP(prod_tanh_##K) BD_DECLARE_RECOMPUTE(prod_tanh_##K)
BD_ARITY_LIST(BD_DECL_ARITY)

bool bd_bwd_has_signature(int M, int nf, int nr, int nc, int na, uint64_t absent, uint64_t share, int chunks, bool strided);
hipError_t bd_bwd_tiled(int dt, int vec, bool signature, int nf, int nr, int nc, int na, uint64_t absent, uint64_t share,
                        const BwdTiledParams &p, dim3 grid, size_t lds, const Launch &s);
hipError_t bd_bwd_pass2(int dt, const Pass2Params &p, int64_t n_blocks, const Launch &s);
hipError_t bd_bwd_generic(int dt, int kind, const BwdGenericParams &p, int64_t n_blocks, const Launch &s);
hipError_t bd_stream_probe(int n_in, const void *const *in, const int64_t *in_stride, int n_out, void *const *out,
                           const int64_t *out_stride, int64_t n_chunks, bool nt_loads, bool reverse, size_t lds_bytes,
                           const Launch &s);

namespace {

struct OpDesc {
  const char *name;
  int n_args, n_out;
  uint32_t nondiff;
  int n_branches;
  const int8_t *alias;  // per plane: own index, index of an identical earlier plane, or -1 (always zero); nullptr: all distinct
  hipError_t (*tiled)(int, int, const FwdTiledParams &, dim3, const Launch &);
  hipError_t (*generic)(int, const FwdGenericParams &, dim3, const Launch &);
  hipError_t (*recompute)(int, int, int, const BwdTiledParams &, const RecomputeArgs &, dim3, size_t, const Launch &);  // may be null
  uint64_t (*recompute_pattern)();
  bool strided;  // the tiled forward kernel is also built for views with row strides of their own
};

// HM-LSTM update, planes (c' then h') x (f i o g c h b_f b_i b_o b_g): a bias enters only through
// its gate's pre-activation, so its plane equals the gate's; c' never depends on o, h, b_o.
const int8_t kAliasHmLstm[20] = {0, 1, -1, 3, 4, -1, 0, 1, -1, 3, 10, 11, 12, 13, 14, 15, 10, 11, 12, 13};
// branchy5 (A B r s t): the threshold t only appears in the predicate
const int8_t kAliasBranchy5[5] = {0, 1, 2, 3, -1};

#define BD_OP_ROW(NAME, N, M, NONDIFF, NBR) \
  {#NAME, N, M, NONDIFF, NBR, nullptr, bd_fwd_tiled_##NAME, bd_fwd_generic_##NAME, bd_bwdr_tiled_##NAME, bd_bwdr_pattern_##NAME, true},
#define BD_OP_ROW_A(NAME, N, M, NONDIFF, NBR, ALIAS) \
  {#NAME, N, M, NONDIFF, NBR, ALIAS, bd_fwd_tiled_##NAME, bd_fwd_generic_##NAME, bd_bwdr_tiled_##NAME, bd_bwdr_pattern_##NAME, true},
#define BD_ARITY_ROW(K) \
  {"prod_tanh_" #K, K, 1, 0u, K + 1, nullptr, bd_fwd_tiled_prod_tanh_##K, bd_fwd_generic_prod_tanh_##K, bd_bwdr_tiled_prod_tanh_##K, \
   bd_bwdr_pattern_prod_tanh_##K, false},
const OpDesc kOps[] = {
    BD_OP_ROW_A(hmlstm_update, 12, 2, (1u << 6) | (1u << 7), 3, kAliasHmLstm)
    BD_OP_ROW(tanh_xy_b, 3, 1, 0u, 1)
    BD_OP_ROW_A(branchy5, 5, 1, 0u, 2, kAliasBranchy5)
    BD_OP_ROW(update_c, 6, 1, (1u << 4) | (1u << 5), 3)
    BD_OP_ROW(cos_x, 1, 1, 0u, 1)
    BD_OP_ROW(scale_xt, 2, 1, 0u, 1)
    BD_OP_ROW(pair3, 3, 2, 0u, 1)
    BD_OP_ROW(linear12, 12, 2, (1u << 6) | (1u << 7), 1)
    BD_OP_ROW(elementary4, 1, 4, 0u, 1)
    BD_ARITY_LIST(BD_ARITY_ROW)
};
constexpr int kNumOps = (int)(sizeof(kOps) / sizeof(kOps[0]));

// ---- per-call options ------------------------------------------------------------------------
using Opt = bcast_dual_options;
// what a forward launch of more than 1 GiB of output writes plainly at the end of its walk when fwd_keep_mib is automatic
constexpr int kFwdKeepMiB = 256;
// full-shape gradient bytes of one backward call from which on they are written with the nontemporal hint
constexpr int64_t kNtGradientBytes = (int64_t)256 << 20;
// plane bytes (written by a forward launch, read by a backward one) up to which the whole step fits the memory-side cache
constexpr int64_t kSmallStepBytes = (int64_t)128 << 20;

void default_options(Opt &o) {
  std::memset(&o, 0, sizeof o);
  o.struct_size = (uint32_t)sizeof(Opt);
  o.nontemporal_stores = 3;
  o.max_vector_bytes = 16;
  o.reverse_tiles = 2;
  o.interleave_rows = 1;
  o.col_chunks = 1;
  o.fwd_lds_kib = -1;
  o.narrow_tiles = 1;
  o.ragged_rows = 1;
  o.probe_nt_loads = 1;
  o.fwd_keep_mib = -1;
  o.bwd_nt_min_mib = -1;
}

// NULL: the defaults; otherwise a checked copy
int resolve_options(const bcast_dual_options *in, Opt &o) {
  if (in == nullptr) {
    default_options(o);
    return BCAST_OK;
  }
  if (in->struct_size != sizeof(Opt)) return BCAST_ERR_BAD_OPTION;
  o = *in;
  auto in_range = [](int32_t v, int32_t lo, int32_t hi) { return v >= lo && v <= hi; };
  const bool ok = in_range(o.bwd_row_steps, 0, 512) && in_range(o.nontemporal_stores, 0, 3) && in_range(o.force_generic, 0, 1) &&
                  (o.max_vector_bytes == 4 || o.max_vector_bytes == 8 || o.max_vector_bytes == 16) && in_range(o.runtime_table, 0, 1) &&
                  in_range(o.reverse_tiles, 0, 2) && in_range(o.interleave_rows, 0, 1) && in_range(o.xcd_order, 0, 1) &&
                  in_range(o.col_chunks, 0, 1) && in_range(o.fwd_lds_kib, -1, 64) && in_range(o.bwd_lds_kib, 0, 64) &&
                  in_range(o.narrow_tiles, 0, 1) && in_range(o.ragged_rows, 0, 1) && in_range(o.probe_nt_loads, 0, 1) &&
                  in_range(o.probe_lds_kib, 0, 64) && in_range(o.fwd_keep_mib, -1, 1 << 20) && in_range(o.bwd_nt_min_mib, -1, 1 << 20) &&
                  ((o.start_event == nullptr) == (o.stop_event == nullptr));
  return ok ? BCAST_OK : BCAST_ERR_BAD_OPTION;
}

// stream and (for the call's main-pass kernel only) the caller's event pair
Launch on_stream(void *stream, const Opt *timed = nullptr) {
  return Launch{static_cast<hipStream_t>(stream), timed ? static_cast<hipEvent_t>(timed->start_event) : nullptr,
                timed ? static_cast<hipEvent_t>(timed->stop_event) : nullptr};
}

// A failed launch is reported with the runtime's own words on stderr: the status code alone
// cannot say why.
int launch_status(hipError_t e) {
  if (e == hipSuccess) return BCAST_OK;
  std::fprintf(stderr, "bcast_dual: kernel launch failed: %s\n", hipGetErrorString(e));
  return BCAST_ERR_LAUNCH_FAILED;
}

// ---- small helpers ---------------------------------------------------------------------------
inline size_t elem_size(int dt) { return dt == BCAST_F32 ? 4 : 8; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int ilog2_ceil(int64_t x) {
  int l = 0;
  while (((int64_t)1 << l) < x) ++l;
  return l;
}
inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

using Dims = std::array<int64_t, BCAST_MAX_DIMS>;

// A view padded to the common rank D with trailing size-1 dims.
struct PView {
  void *p = nullptr;
  Dims shape{{1, 1, 1, 1}};
  Dims stride{{0, 0, 0, 0}};
};

int check_view(const bcast_tensor &t, size_t esize, bool allow_null, bool written, PView &out) {
  if (t.ndim < 0 || t.ndim > BCAST_MAX_DIMS) return BCAST_ERR_RANK_TOO_HIGH;
  bool empty = false;
  for (int d = 0; d < t.ndim; ++d) empty |= (t.shape[d] == 0);
  if (t.data == nullptr && !allow_null && !empty) return BCAST_ERR_NULL_POINTER;
  if (reinterpret_cast<uintptr_t>(t.data) % esize != 0) return BCAST_ERR_MISALIGNED;
  out.p = t.data;
  // Nothing a kernel could address: more than 2^40 elements, or an element 2^44 elements or more
  // from the view's start (checked in 128 bits, so that absurd extents and strides cannot wrap
  // the 64-bit index arithmetic further down).
  unsigned __int128 count = 1, reach = 0;
  for (int d = 0; d < t.ndim; ++d) {
    if (t.shape[d] < 0) return BCAST_ERR_SHAPE_MISMATCH;
    out.shape[d] = t.shape[d];
    out.stride[d] = t.shape[d] == 1 ? 0 : t.stride[d];
    if (out.stride[d] < 0) return BCAST_ERR_BAD_STRIDE;
    count *= (unsigned __int128)t.shape[d];
    if (count > ((unsigned __int128)1 << 40)) return BCAST_ERR_SHAPE_MISMATCH;
    if (t.shape[d] > 1) reach += (unsigned __int128)(t.shape[d] - 1) * (unsigned __int128)out.stride[d];
    if (reach >= ((unsigned __int128)1 << 44)) return BCAST_ERR_BAD_STRIDE;
  }
  if (written && t.data != nullptr) {
    // every written element must have its own address
    std::array<std::pair<int64_t, int64_t>, BCAST_MAX_DIMS> se;
    int n = 0;
    for (int d = 0; d < t.ndim; ++d)
      if (t.shape[d] > 1) se[n++] = {t.stride[d], t.shape[d]};
    std::sort(se.begin(), se.begin() + n);
    int64_t reach = 0;
    for (int q = 0; q < n; ++q) {
      if (se[q].first <= reach) return BCAST_ERR_BAD_STRIDE;
      reach += (se[q].second - 1) * se[q].first;
    }
  }
  return BCAST_OK;
}

// The merged problem: dims of extent 1 dropped, the rest ordered by the key tensor's
// stride (largest first) and adjacent dims fused wherever every tensor allows it.
struct Canon {
  int nd = 0;
  Dims shape{{1, 1, 1, 1}};
  int64_t E = 1;
  std::vector<Dims> strides;  // per tensor, merged dims, outermost first
};

constexpr int64_t kMaxFused = (int64_t)1 << 28;
void canonicalize(int D, const Dims &U, const std::vector<Dims> &eff, int key, Canon &c) {
  int order[BCAST_MAX_DIMS], n_order = 0;
  for (int d = 0; d < D; ++d)
    if (U[d] > 1) order[n_order++] = d;
  std::stable_sort(order, order + n_order, [&](int a, int b) { return eff[key][a] > eff[key][b]; });
  // merged dims so far: extents in shp, per-tensor strides in cur (no allocation per tensor:
  // this runs on every call)
  const size_t nt = eff.size();
  int64_t shp[BCAST_MAX_DIMS];
  int n = 0;
  std::vector<Dims> &cur = c.strides;
  cur.assign(nt, Dims{{0, 0, 0, 0}});
  for (int q = 0; q < n_order; ++q) {
    const int d = order[q];
    // a fused dim stays below 2^28 elements: the tiled kernels address a row with 32-bit byte offsets
    bool merge = n > 0 && shp[n - 1] <= kMaxFused / U[d];
    if (merge)
      for (size_t t = 0; t < nt && merge; ++t) merge = (cur[t][n - 1] == eff[t][d] * U[d]);
    if (merge) {
      shp[n - 1] *= U[d];
      for (size_t t = 0; t < nt; ++t) cur[t][n - 1] = eff[t][d];
    } else {
      shp[n] = U[d];
      for (size_t t = 0; t < nt; ++t) cur[t][n] = eff[t][d];
      ++n;
    }
  }
  // one dim longer than that (a long vector, or dims the caller had fused already): taken as rows
  // of equal length if a power of two up to 2^16 divides it suitably
  if (n == 1 && shp[0] > kMaxFused)
    for (int64_t f = 2; f <= 65536; f *= 2)
      if (shp[0] % f == 0 && shp[0] / f <= kMaxFused) {
        const int64_t inner = shp[0] / f;
        shp[0] = f;
        shp[1] = inner;
        n = 2;
        for (size_t t = 0; t < nt; ++t) cur[t] = Dims{{cur[t][0] * inner, cur[t][0], 0, 0}};
        break;
      }
  c.nd = n;
  c.E = 1;
  c.shape = Dims{{1, 1, 1, 1}};
  for (int d = 0; d < n; ++d) {
    c.shape[d] = shp[d];
    c.E *= shp[d];
  }
}

// slices / rows / columns of a merged problem of rank <= 3 (a problem of three dims is a batch of O
// two-dim slices for the tiled kernels), and one tensor's strides in it
struct Shape2 {
  int64_t O = 1, R = 1, C = 1;
};
inline Shape2 shape2(const Canon &c) {
  Shape2 s;
  if (c.nd == 1) s.C = c.shape[0];
  if (c.nd == 2) { s.R = c.shape[0]; s.C = c.shape[1]; }
  if (c.nd == 3) { s.O = c.shape[0]; s.R = c.shape[1]; s.C = c.shape[2]; }
  return s;
}
inline TView tview(const Canon &c, size_t t, void *p) {
  TView v{p, 0, 0, 0};
  if (c.nd == 1) v.sc = c.strides[t][0];
  if (c.nd == 2) { v.sr = c.strides[t][0]; v.sc = c.strides[t][1]; }
  if (c.nd == 3) { v.so = c.strides[t][0]; v.sr = c.strides[t][1]; v.sc = c.strides[t][2]; }
  return v;
}
inline SView sview(const Canon &c, size_t t, void *p) {
  const TView v = tview(c, t, p);
  return SView{v.p, v.sr, v.so};
}
inline GView gview(const Canon &c, size_t t, void *p) {
  GView v{p, {0, 0, 0, 0}};
  for (int d = 0; d < c.nd; ++d) v.s[d] = c.strides[t][d];
  return v;
}

// Row strides of the views that vary along rows and columns.  Returns the stride they share,
// -1 if they differ from one another (each view is then addressed with its own), or -2 if the
// rows that one block takes in one step (up to 256 when rows are shorter than 1024 elements,
// else one) span 4 GiB or more of some view: lanes address a row step with 32-bit byte offsets
// from its first row.  The size of a view as a whole is not limited by this.
// Views [0, n_streamed) are the ones a kernel streams row by row with the common stride (the
// adjoints and planes of a backward call): one of them that repeats a single row (row stride 0
// with more than one row -- an expanded view) has a row stride of its own like any other and
// breaks the uniformity.  Views past that index with row stride 0 are row vectors, which the
// kernels address apart, and are skipped.
// With three dims the same holds for the strides between slices: `outer` receives the one the
// views share (views that repeat one slice break the uniformity among the streamed ones like
// views that repeat one row).
int64_t common_row_stride(const Canon &c, const std::vector<PView> &v, const Shape2 &s2, size_t es, size_t n_streamed, int64_t *outer) {
  *outer = 0;
  if (s2.R == 1 && s2.O == 1) return s2.C * es > 0xffffffffULL ? -2 : 0;
  int64_t sr = -1, so = -1;
  bool uniform = true;
  const int64_t rows_in_step = std::min<int64_t>(s2.R, s2.C >= 1024 ? 1 : kBlock);
  for (size_t t = 0; t < v.size(); ++t) {
    if (!v[t].p) continue;
    const TView tv = tview(c, t, nullptr);
    if (tv.sc == 0) continue;
    const unsigned __int128 last = ((unsigned __int128)(rows_in_step - 1) * tv.sr + s2.C) * es;
    if (last > 0xffffffffULL) return -2;
    if (tv.sr == 0 && s2.R > 1) {  // a row vector (of each slice): addressed apart, unless it is a streamed view
      if (t < n_streamed) uniform = false;
      continue;
    }
    if (tv.so == 0 && s2.O > 1) {  // the same rows for every slice: rows with a stride, slices without
      uniform = false;
      continue;
    }
    if (sr < 0) {
      sr = tv.sr;
      so = tv.so;
    } else if (sr != tv.sr || so != tv.so) {
      uniform = false;
    }
  }
  if (!uniform) return -1;
  *outer = so < 0 ? 0 : so;
  return sr < 0 ? 0 : sr;  // no such view: the offset is never used
}

// Rows of 1024 elements and more are normally taken one per block step (common_row_stride counts
// on that); up to four per step are possible only if four rows of every view still span less than 4 GiB.
bool narrow_tiles_ok(const Canon &c, const std::vector<PView> &v, const Shape2 &s2, size_t es) {
  for (size_t t = 0; t < v.size(); ++t) {
    if (!v[t].p) continue;
    const TView tv = tview(c, t, nullptr);
    if (tv.sc == 0) continue;
    if (((unsigned __int128)3 * tv.sr + s2.C) * es > 0xffffffffULL) return false;
  }
  return true;
}

struct Geometry {
  int vec = 1, log2_tx = 0, steps = 1;
  int64_t n_ct = 1, n_rt = 1;
};

// Lanes along the columns: the smallest power of two covering the row, at most a block.  A row
// longer than a block's 256 lanes is cut into column tiles; a last tile with few lanes in use
// still costs whole blocks (4096 x 1028 fp32, 257 vectors per row, took 265 us per step against
// 154 us for 4096 x 1024), so 64 or 128 lanes per row (4 or 2 rows per block step) are taken
// instead where that pads the row less -- a wavefront still covers 1 KiB of a row.
void tile_columns(int64_t C, int vec, bool narrow_ok, const Opt &o, Geometry &g) {
  const int64_t units = ceil_div(C, vec);
  g.log2_tx = std::min(8, ilog2_ceil(units));
  if (units > 256 && narrow_ok && o.narrow_tiles != 0) {
    const int64_t padded256 = ceil_div(units, 256) * 256;
    int64_t best = padded256;
    int best_l = 8;
    for (int l = 7; l >= 6; --l) {  // ties go to the wider tile
      const int64_t padded = ceil_div(units, (int64_t)1 << l) << l;
      if (padded < best) {
        best = padded;
        best_l = l;
      }
    }
    // narrow tiles cost about a tenth themselves (shorter runs per row): 16384 x 4100, 80 % full at
    // 256 lanes and 94 % at 64, ran 1.86 against 1.69 ms in the reverse pass with them
    if (best * 5 <= padded256 * 4) g.log2_tx = best_l;
  }
  g.n_ct = ceil_div(units, (int64_t)1 << g.log2_tx);
}
// false if the problem needs more blocks than one launch can have
bool tile_rows(int64_t R, int steps, Geometry &g) {
  const int TY = kBlock >> g.log2_tx;
  const int64_t row_steps = ceil_div(R, TY);
  steps = (int)std::max<int64_t>(1, std::min<int64_t>(steps, row_steps));
  g.steps = steps;
  g.n_rt = ceil_div(row_steps, steps);
  return g.n_ct <= 0x7fffffffLL && g.n_rt <= 0x7fffffffLL / g.n_ct;
}
// enough blocks to fill 256 CUs several times over, a few rows per block to amortise
// the per-block set-up
int auto_steps(int64_t R, const Geometry &g, int max_steps) {
  const int TY = kBlock >> g.log2_tx;
  const int64_t row_steps = ceil_div(R, TY);
  const int64_t want_blocks = 256 * 16;
  int64_t s = (row_steps * g.n_ct) / want_blocks;
  return (int)std::max<int64_t>(1, std::min<int64_t>(s, max_steps));
}

// Rows that the 16-byte vector does not fit (a length that is no multiple of it, a start or a row
// stride off its boundary; `vw`: what the aligned kernels could take) go to the kernels that read
// unaligned vectors and finish every row element by element.  Those exist for the widest vector
// and views with one common row stride; a row must hold one whole vector.
bool ragged_rows_ok(int vw, bool uniform_stride, const Shape2 &s2, size_t es, const Opt &o) {
  const int widest = (int)(16 / es);
  return o.ragged_rows != 0 && o.max_vector_bytes >= 16 && vw < widest && uniform_stride && s2.C >= widest;
}

// Whether a lane of the generic kernels may take `vw` consecutive elements of the innermost dim of
// view `t` as one vector: the view runs contiguously along that dim (or, where `may_be_constant`,
// does not vary along it), starts on a vector boundary and keeps to one with every outer stride.
bool generic_vector_ok(const Canon &c, size_t t, const void *ptr, int vw, size_t es, bool may_be_constant) {
  const int in = c.nd - 1;
  const int64_t s_in = c.strides[t][in];
  if (s_in == 0) return may_be_constant;
  if (s_in != 1 || reinterpret_cast<uintptr_t>(ptr) % (vw * es) != 0) return false;
  for (int d = 0; d < in; ++d)
    if (c.strides[t][d] % vw != 0) return false;
  return true;
}

// ---- forward planning ----------------------------------------------------------------------------
struct FwdPlan {
  bcast_plan_info info{};
  bool tiled = false;
  FwdTiledParams tp{};
  FwdGenericParams gp{};
  dim3 grid{1, 1, 1};
};

int plan_forward(int32_t op_id, int dt, int32_t n_args, const bcast_tensor *args, int32_t n_out,
                 const bcast_tensor *outs, const bcast_tensor *partials, const uint8_t *branch_id,
                 const Opt &o, FwdPlan &plan) {
  if (op_id < 0 || op_id >= kNumOps) return BCAST_ERR_INVALID_OP;
  if (dt != BCAST_F32 && dt != BCAST_F64) return BCAST_ERR_BAD_DTYPE;
  const OpDesc &op = kOps[op_id];
  if (n_args != op.n_args || n_out != op.n_out) return BCAST_ERR_BAD_ARG_COUNT;
  if (args == nullptr || outs == nullptr) return BCAST_ERR_NULL_POINTER;
  const size_t es = elem_size(dt);
  const int N = op.n_args, M = op.n_out;
  const int ND = N - __builtin_popcount(op.nondiff);
  const int n_planes = partials ? M * ND : 0;

  std::vector<PView> v(N + M + n_planes);
  int D = 0;
  for (int j = 0; j < N; ++j) {
    if (int rc = check_view(args[j], es, false, false, v[j])) return rc;
    D = std::max(D, args[j].ndim);
  }
  for (int i = 0; i < M; ++i) {
    if (int rc = check_view(outs[i], es, false, true, v[N + i])) return rc;
    D = std::max(D, outs[i].ndim);
  }
  for (int k = 0; k < n_planes; ++k) {
    if (int rc = check_view(partials[k], es, true, true, v[N + M + k])) return rc;
    D = std::max(D, partials[k].ndim);
  }
  // unified shape: per dim the extent that is not 1 (all such must agree)
  Dims U{{1, 1, 1, 1}};
  for (int d = 0; d < D; ++d)
    for (int j = 0; j < N; ++j) {
      const int64_t s = v[j].shape[d];
      if (s == 1) continue;
      if (U[d] == 1) U[d] = s;
      else if (U[d] != s) return BCAST_ERR_SHAPE_MISMATCH;
    }
  bool E0 = false;
  for (int d = 0; d < D; ++d) E0 |= (U[d] == 0);
  for (size_t t = N; t < v.size(); ++t)
    if ((v[t].p || (E0 && t < (size_t)(N + M))) && v[t].shape != U) return BCAST_ERR_OUTPUT_SHAPE_MISMATCH;

  int64_t E = 1;
  for (int d = 0; d < D; ++d) E *= U[d];
  plan.info = bcast_plan_info{};
  if (E == 0) return BCAST_OK;

  // Two plane slots may share one view only where the op declares the planes identical;
  // the later slot is then not written a second time.
  std::vector<char> dup(n_planes, 0);
  for (int k = 1; k < n_planes; ++k) {
    if (!v[N + M + k].p) continue;
    for (int j = 0; j < k; ++j) {
      if (v[N + M + j].p != v[N + M + k].p) continue;
      const bool same_view = v[N + M + j].stride == v[N + M + k].stride;
      if (!same_view || !op.alias || op.alias[k] < 0 || op.alias[k] != op.alias[j]) return BCAST_ERR_BAD_STRIDE;
      dup[k] = 1;
      break;
    }
  }

  // effective strides: stride 0 wherever an argument's dim is 1 (virtual copy)
  std::vector<Dims> eff;
  eff.reserve(v.size() + 1);
  for (auto &pv : v) eff.push_back(pv.p ? pv.stride : v[N].stride);  // absent planes never block a merge
  const bool want_branch = branch_id != nullptr;
  if (want_branch) {  // row-major over the unified shape as given
    Dims bs{{0, 0, 0, 0}};
    int64_t acc = 1;
    for (int d = D - 1; d >= 0; --d) {
      bs[d] = U[d] > 1 ? acc : 0;
      acc *= U[d];
    }
    eff.push_back(bs);
  }
  Canon c;
  canonicalize(D, U, eff, N /* key: the first output */, c);
  plan.info.ndim = c.nd;
  for (int d = 0; d < c.nd; ++d) plan.info.shape[d] = c.shape[d];

  bool tiled = (c.nd <= 3) && !o.force_generic;
  const Shape2 s2 = shape2(c);
  if (tiled && s2.C > 1) {
    for (int j = 0; j < N && tiled; ++j) {
      const int64_t sc = tview(c, j, nullptr).sc;
      tiled = (sc == 0 || sc == 1);
    }
    for (size_t t = N; t < v.size() && tiled; ++t)
      if (v[t].p) tiled = (tview(c, t, nullptr).sc == 1);
  }
  int64_t fwd_so = 0;
  const int64_t fwd_sr = tiled ? common_row_stride(c, v, s2, es, 0, &fwd_so) : -2;
  // views with row strides of their own: only the ops built for it (the others go generic)
  tiled = tiled && (fwd_sr >= 0 || (fwd_sr == -1 && op.strided));
  plan.tiled = tiled;
  if (tiled) {
    FwdTiledParams &p = plan.tp;
    p.uniform_stride = fwd_sr >= 0;
    p.row_stride = fwd_sr >= 0 ? fwd_sr : 0;
    p.outer_stride = fwd_sr >= 0 ? fwd_so : 0;
    p.O = s2.O;
    p.R = s2.R;
    p.C = s2.C;
    // widest vector (16 bytes per lane at most) that every vector-accessed view allows
    int vw = (int)(std::max<int>(o.max_vector_bytes, (int)es) / es);
    for (; vw > 1; vw /= 2) {
      bool vec_ok = (s2.C % vw == 0);
      for (size_t t = 0; t < v.size() && vec_ok; ++t) {
        if (!v[t].p) continue;
        const TView tv = tview(c, t, v[t].p);
        if (tv.sc == 0 && s2.C > 1) continue;  // a broadcast load: one element
        vec_ok = (reinterpret_cast<uintptr_t>(tv.p) % (vw * es) == 0) && (s2.R == 1 || tv.sr % vw == 0) && (s2.O == 1 || tv.so % vw == 0);
      }
      if (vec_ok) break;
    }
    if (!p.uniform_stride && vw != (int)(16 / es)) vw = 1;  // those kernels exist for the widest vector and for 1
    p.ragged = ragged_rows_ok(vw, p.uniform_stride != 0, s2, es, o);
    if (p.ragged) vw = (int)(16 / es);
    Geometry g;
    g.vec = vw;
    tile_columns(s2.C, g.vec, narrow_tiles_ok(c, v, s2, es), o, g);
    if (!tile_rows(s2.R, 1, g)) return BCAST_ERR_LAUNCH_FAILED;  // the forward kernel has no row loop
    if (g.n_ct * g.n_rt > 0x7fffffffLL / s2.O) return BCAST_ERR_LAUNCH_FAILED;
    p.tiles_per_slice = g.n_ct * g.n_rt;
    p.n_ct = g.n_ct;
    p.log2_tx = g.log2_tx;
    p.xcd_remap = o.xcd_order != 0 && (s2.O * g.n_ct * g.n_rt) % 8 == 0;
    p.has_partials = n_planes > 0;
    for (int j = 0; j < N; ++j) {
      const TView tv = tview(c, j, v[j].p);
      p.arg_p[j] = tv.p;
      p.arg_sr[j] = tv.sr;
      p.arg_so[j] = tv.so;
      // (a problem of one row has no row vectors: nothing is read by a second row of blocks, and the
      // kernel keeps the streaming loads of full-shape arguments for it)
      if (tv.sr == 0 && s2.R > 1) p.row_invariant |= 1u << j;
      if (tv.sc == 0) p.col_invariant |= 1u << j;
    }
    for (int i = 0; i < M; ++i) {
      p.out_p[i] = v[N + i].p;
      p.out_sr[i] = tview(c, N + i, nullptr).sr;
      p.out_so[i] = tview(c, N + i, nullptr).so;
    }
    for (int k = 0; k < n_planes; ++k) {
      p.part_p[k] = dup[k] ? nullptr : v[N + M + k].p;
      p.part_sr[k] = tview(c, N + M + k, nullptr).sr;
      p.part_so[k] = tview(c, N + M + k, nullptr).so;
    }
    // A launch that mostly writes (two or more planes read, at least 2.5 written for each) runs fastest
    // with three blocks, twelve wavefronts, per CU: measured 75 against 81 us on the HM-LSTM
    // update (7 read, 22 written), 355 against 382 us on 8192 x 8192 branchy5 (2 read, 6 written),
    // and slower again with two blocks.  Dynamic LDS that the kernel never touches (48 of the
    // CU's 160 KiB per block) sets that limit.  Balanced and read-heavy launches, the
    // values-only one among them, want every wavefront they can get and are left alone.
    int planes_read = 0, planes_written = M;
    for (int j = 0; j < N; ++j) planes_read += !((p.row_invariant | p.col_invariant) >> j & 1u);
    for (int k = 0; k < n_planes; ++k) planes_written += p.part_p[k] != nullptr;
    // fp64 runs best with four blocks (cfg 4 in fp64: 722 against 750 us with three, 770 with no limit).
    const int lds_kib = o.fwd_lds_kib >= 0 ? o.fwd_lds_kib : (es == 8 ? 40 : 48);
    p.lds_bytes = planes_read >= 2 && 2 * planes_written >= 5 * planes_read ? lds_kib * 1024 : 0;
    // Nontemporal stores for everything but the tail of what the launch writes (see fwd_keep_mib): the
    // tail, kept in the caches, is what a reverse pass walking last to first reads first.
    {
      const int64_t n_tiles = s2.O * g.n_ct * g.n_rt;
      const int64_t tile_bytes = (int64_t)planes_written * (kBlock >> g.log2_tx) * ((int64_t)g.vec << g.log2_tx) * (int64_t)es;
      // Automatic, by how what is written compares with the caches (32 MB of L2, 256 MB memory-side):
      //  - up to 128 MiB (a whole forward + reverse step then fits the memory-side cache): hint everywhere; the data
      //    reaches that cache either way, and plain stores leave it to the end of the kernel to write the L2 back
      //    (HM-LSTM 2048 x 256, 46 MB written: 27.0 -> 23.7 us per step with the reverse pass doing the same);
      //  - up to 1 GiB: plain everywhere; the memory-side cache absorbs the writes faster than memory takes them
      //    and the reverse pass finds most of them there (4096 x 1024, 369 MB: 74 us plain, 94 us with the hint);
      //  - beyond: hint, except for the last 256 MiB, which the reverse pass reads first (8192 x 8192 branchy5,
      //    1.6 GB: forward 363 -> 340 us).
      const int64_t total = n_tiles * tile_bytes;
      const int64_t auto_keep = total <= kSmallStepBytes ? 0 : total <= ((int64_t)1 << 30) ? total : (int64_t)kFwdKeepMiB << 20;
      const int64_t keep_bytes = o.fwd_keep_mib >= 0 ? (int64_t)o.fwd_keep_mib << 20 : auto_keep;
      const int64_t keep_tiles = (keep_bytes + tile_bytes - 1) / tile_bytes;
      p.nt_tiles = (o.nontemporal_stores & 1) && keep_tiles < n_tiles ? (uint32_t)(n_tiles - keep_tiles) : 0u;
    }
    if (want_branch) {
      const TView tv = tview(c, v.size(), const_cast<uint8_t *>(branch_id));
      p.branch_p = static_cast<uint8_t *>(tv.p);
      p.branch_sr = tv.sr;
      p.branch_sc = tv.sc;
      p.branch_so = tv.so;
    }
    plan.grid = dim3((unsigned)(s2.O * g.n_ct * g.n_rt), 1, 1);
    plan.info.path = 1;
    plan.info.vec = g.vec;
    plan.info.ragged = p.ragged;
    plan.info.uniform_stride = p.uniform_stride;
    plan.info.nontemporal_tiles = p.nt_tiles;
    plan.info.tx = 1 << g.log2_tx;
    plan.info.ty = kBlock >> g.log2_tx;
    plan.info.rows_per_block = plan.info.ty * g.steps;
    plan.info.grid_x = g.n_ct;
    plan.info.grid_y = g.n_rt * s2.O;
  } else {
    FwdGenericParams &p = plan.gp;
    p.nd = c.nd;
    for (int d = 0; d < BCAST_MAX_DIMS; ++d) p.shape[d] = d < c.nd ? c.shape[d] : 1;
    p.E = c.E;
    for (int j = 0; j < N; ++j) p.arg[j] = gview(c, j, v[j].p);
    for (int i = 0; i < M; ++i) p.out[i] = gview(c, N + i, v[N + i].p);
    for (int k = 0; k < M * ND; ++k)
      p.part[k] = (k < n_planes && !dup[k]) ? gview(c, N + M + k, v[N + M + k].p) : GView{nullptr, {0, 0, 0, 0}};
    p.branch = want_branch ? gview(c, v.size(), const_cast<uint8_t *>(branch_id)) : GView{nullptr, {0, 0, 0, 0}};
    // 16-byte vectors along the innermost dim where every view allows them (ops built in every variant)
    int gv = op.strided && c.nd >= 1 ? (int)(std::max<int>(o.max_vector_bytes, (int)es) / es) : 1;
    if (gv != (int)(16 / es) || c.shape[c.nd - 1] % gv != 0) gv = 1;
    for (size_t t = 0; t < v.size() && gv > 1; ++t)
      if (v[t].p && !(t >= (size_t)(N + M) && dup[t - N - M]) && !generic_vector_ok(c, t, v[t].p, gv, es, t < (size_t)N)) gv = 1;
    p.vec = gv;
    const int64_t blocks = ceil_div(c.E / gv, kBlock);
    if (blocks > 0x7fffffffLL) return BCAST_ERR_LAUNCH_FAILED;
    plan.grid = dim3((unsigned)blocks, 1, 1);
    plan.info.path = 2;
    plan.info.vec = gv;
    plan.info.tx = kBlock;
    plan.info.ty = 1;
    plan.info.rows_per_block = 1;
    plan.info.grid_x = blocks;
    plan.info.grid_y = 1;
  }
  plan.info.n_launches = 1;
  return BCAST_OK;
}

// ---- backward planning ---------------------------------------------------------------------------
constexpr size_t kLdsBudget = 48 * 1024;

struct BwdPlan {
  bcast_plan_info info{};
  bool tiled = false;
  int vec = 1;
  bool signature = false;          // a kernel compiled for exactly this mix of gradient classes exists
  int n_cls[4] = {0, 0, 0, 0};     // gradients per class: full, row-sum, col-sum, all-sum
  uint64_t absent = 0;             // bit e*M + i: plane i of table entry e is absent
  uint64_t share = 0;              // 4 bits per table entry e: s + 1 if e has the very planes of an earlier entry s
  RecomputeArgs ra{};              // recompute mode only
  int fixed_pattern = 0;           // recompute mode: 1 = the call has the op's compiled-in broadcast pattern, 2 = that pattern transposed
  std::vector<BwdTiledParams> main;  // usually one launch
  std::vector<size_t> main_lds;
  dim3 grid{1, 1, 1};
  Pass2Params p2{};
  int64_t p2_blocks = 0;
  std::vector<std::pair<int, BwdGenericParams>> generic;  // (0 elementwise / 1 reduction / 2 sum of partial sums, params)
  std::vector<int64_t> generic_blocks;
  size_t ws_bytes = 0;
};

// With `rop` set this plans the recompute-in-reverse call instead: there are no planes, the
// op's n_args arguments are read (and must broadcast to the adjoints' shape), and only the
// tiled kernels are available.
int plan_backward(int dt, int32_t n_out, const bcast_tensor *adjoints, const bcast_tensor *partials,
                  int32_t n_grads, const bcast_tensor *grads, const Opt &o, BwdPlan &plan, const OpDesc *rop = nullptr,
                  const bcast_tensor *args = nullptr) {
  if (dt != BCAST_F32 && dt != BCAST_F64) return BCAST_ERR_BAD_DTYPE;
  if (n_out < 1 || n_out > BCAST_MAX_OUTS || n_grads < 1 || n_grads > BCAST_MAX_ARGS ||
      n_out * n_grads > BCAST_MAX_PLANES)
    return BCAST_ERR_BAD_ARG_COUNT;
  if (adjoints == nullptr || (partials == nullptr && !rop) || grads == nullptr || (rop && !args))
    return BCAST_ERR_NULL_POINTER;
  const int NA = rop ? rop->n_args : 0;
  const size_t es = elem_size(dt);
  const size_t as = dt == BCAST_F32 ? 8 : 16;  // accumulator bytes
  const int M = n_out, ND = n_grads;
  std::vector<PView> v(M + M * ND + ND + NA);
  const size_t a0 = M + M * ND + ND;  // first argument view (recompute mode)
  int D = 0;
  for (int i = 0; i < M; ++i) {
    if (int rc = check_view(adjoints[i], es, false, false, v[i])) return rc;
    D = std::max(D, adjoints[i].ndim);
  }
  for (int k = 0; k < M * ND && !rop; ++k) {
    if (int rc = check_view(partials[k], es, true, false, v[M + k])) return rc;
    D = std::max(D, partials[k].ndim);
  }
  for (int j = 0; j < NA; ++j) {
    if (int rc = check_view(args[j], es, false, false, v[a0 + j])) return rc;
    D = std::max(D, args[j].ndim);
  }
  for (int j = 0; j < ND; ++j) {
    if (int rc = check_view(grads[j], es, true, true, v[M + M * ND + j])) return rc;
    D = std::max(D, grads[j].ndim);
  }
  const Dims U = v[0].shape;
  for (int t = 0; t < M + M * ND; ++t)
    if (v[t].p && v[t].shape != U) return BCAST_ERR_OUTPUT_SHAPE_MISMATCH;
  for (int j = 0; j < ND; ++j)
    for (int d = 0; d < BCAST_MAX_DIMS && v[M + M * ND + j].p; ++d) {
      const int64_t s = v[M + M * ND + j].shape[d];
      if (s != U[d] && s != 1) return BCAST_ERR_OUTPUT_SHAPE_MISMATCH;
    }
  for (int j = 0; j < NA; ++j)
    for (int d = 0; d < BCAST_MAX_DIMS; ++d) {
      const int64_t sdim = v[a0 + j].shape[d];
      if (sdim != U[d] && sdim != 1) return BCAST_ERR_SHAPE_MISMATCH;
    }
  if (rop) {  // the arguments are known here: each gradient must have its own argument's shape
    int jd = 0;
    for (int j = 0; j < NA; ++j) {
      if ((rop->nondiff >> j) & 1u) continue;
      if (v[M + M * ND + jd].p && v[M + M * ND + jd].shape != v[a0 + j].shape) return BCAST_ERR_OUTPUT_SHAPE_MISMATCH;
      ++jd;
    }
  }
  int64_t E = 1;
  for (int d = 0; d < BCAST_MAX_DIMS; ++d) E *= U[d];
  plan.info = bcast_plan_info{};
  if (E == 0) return BCAST_OK;

  std::vector<Dims> eff;
  for (auto &pv : v) eff.push_back(pv.stride);
  for (int k = 0; k < M * ND; ++k)
    if (!v[M + k].p) eff[M + k] = eff[0];  // absent planes never block a merge
  for (int j = 0; j < ND; ++j)
    if (!v[M + M * ND + j].p) eff[M + M * ND + j] = eff[0];
  Canon c;
  (void)D;
  canonicalize(BCAST_MAX_DIMS, U, eff, 0 /* key: the first adjoint */, c);
  plan.info.ndim = c.nd;
  for (int d = 0; d < c.nd; ++d) plan.info.shape[d] = c.shape[d];
  const size_t g0 = M + M * ND;

  const Shape2 s2 = shape2(c);
  bool tiled = (c.nd <= 3) && !o.force_generic;
  // class of each gradient in the 2-D picture of one slice, and whether it is summed over the slices too
  std::vector<int> cls(ND, kGradSkip);
  std::vector<char> outer_sum(ND, 0);
  if (tiled) {
    for (int j = 0; j < ND; ++j) {
      if (!v[g0 + j].p) continue;
      const TView tv = tview(c, g0 + j, nullptr);
      const bool rows_red = s2.R > 1 && tv.sr == 0;
      const bool cols_red = s2.C > 1 && tv.sc == 0;
      cls[j] = rows_red ? (cols_red ? kGradAllSum : kGradColSum) : (cols_red ? kGradRowSum : kGradFull);
      outer_sum[j] = s2.O > 1 && tv.so == 0;
      // a gradient with the shape of a slice, summed over the slices only, would need partial sums as
      // large as the problem: left to the generic kernels
      if (cls[j] == kGradFull && outer_sum[j]) tiled = false;
    }
    if (s2.C > 1) {
      for (int t = 0; t < M + M * ND && tiled; ++t)
        if (v[t].p) tiled = (tview(c, t, nullptr).sc == 1);
      for (int j = 0; j < ND && tiled; ++j)
        if (cls[j] == kGradFull) tiled = (tview(c, g0 + j, nullptr).sc == 1);
      for (int j = 0; j < NA && tiled; ++j) {
        const int64_t sc = tview(c, a0 + j, nullptr).sc;
        tiled = (sc == 0 || sc == 1);
      }
    }
  }
  int64_t bwd_sr = -1, bwd_so = 0;
  if (tiled) {
    // reduced gradients are addressed on their own; only full-shape views share the offset
    std::vector<PView> fullv = v;
    for (int j = 0; j < ND; ++j)
      if (cls[j] != kGradFull) fullv[g0 + j].p = nullptr;
    bwd_sr = common_row_stride(c, fullv, s2, es, (size_t)(M + M * ND), &bwd_so);
    tiled = bwd_sr >= -1;  // -1: every view addressed with its own row stride
  }
  const bool uniform_stride = bwd_sr >= 0;
  if (!uniform_stride) bwd_sr = bwd_so = 0;
  plan.tiled = tiled;
  if (rop && (!tiled || (!uniform_stride && !rop->strided))) return BCAST_ERR_UNSUPPORTED;
  if (tiled) {
    int vw = (int)(std::max<int>(o.max_vector_bytes, (int)es) / es);
    for (; vw > 1; vw /= 2) {
      bool vec_ok = (s2.C % vw == 0);
      for (size_t t = 0; t < v.size() && vec_ok; ++t) {
        if (!v[t].p) continue;
        if (t >= g0 && t < a0 && cls[t - g0] != kGradFull) continue;  // reduced gradients are stored by element
        const TView tv = tview(c, t, v[t].p);
        if (t >= a0 && tv.sc == 0 && s2.C > 1) continue;              // a broadcast load: one element
        vec_ok = (reinterpret_cast<uintptr_t>(tv.p) % (vw * es) == 0) && (s2.R == 1 || tv.sr % vw == 0) && (s2.O == 1 || tv.so % vw == 0);
      }
      if (vec_ok) break;
    }
    if (rop && vw != (int)(16 / es)) vw = 1;  // the recompute kernels exist for the widest vector and for 1
    // rows the vector does not fit: kernels that take the vector unaligned
    const bool ragged = ragged_rows_ok(vw, uniform_stride, s2, es, o);
    if (ragged) vw = (int)(16 / es);
    Geometry g;
    g.vec = vw;
    plan.vec = g.vec;
    tile_columns(s2.C, g.vec, narrow_tiles_ok(c, v, s2, es), o, g);
    bool any_rowwise = false;  // sums over rows: worth many rows per block
    int n_rowsum = 0;
    for (int j = 0; j < ND; ++j) {
      any_rowwise |= (cls[j] == kGradColSum || cls[j] == kGradAllSum);
      n_rowsum += (cls[j] == kGradRowSum);
    }
    // the gradient table is ordered by class (full, row-sum, col-sum, all-sum), which is
    // what the signature kernels expect; within a class the argument order is kept
    std::vector<int> order;
    for (int want = kGradFull; want <= kGradAllSum; ++want)
      for (int j = 0; j < ND; ++j)
        if (cls[j] == want) {
          for (int i = 0; i < M; ++i)
            if (v[M + i * ND + j].p == nullptr && order.size() * M + i < 64) plan.absent |= 1ull << (order.size() * M + i);
          order.push_back(j);
          plan.n_cls[want]++;
        }
    // entries whose planes are the very views of an earlier entry (a caller that stores
    // identical planes once): the signature kernels load such planes once
    for (size_t e = 1; rop == nullptr && e < order.size() && e < 16; ++e)
      for (size_t src = 0; src < e; ++src) {
        bool same = true, any = false;
        for (int i = 0; i < M; ++i) {
          const PView &a = v[M + i * ND + order[e]], &b = v[M + i * ND + order[src]];
          same = same && a.p == b.p && (a.p == nullptr || a.stride == b.stride);
          any = any || a.p != nullptr;
        }
        if (same && any) {
          plan.share |= (uint64_t)(src + 1) << (4 * e);
          break;
        }
      }
    // Wide rows with row sums and few planes: a kernel that takes all 2 or 4 column chunks of a
    // row per block finishes the row sums in the main pass (no partial sums, no second pass).
    int chunks = 1;
    if (!rop && uniform_stride && !any_rowwise && n_rowsum > 0 && o.bwd_row_steps == 0 && o.runtime_table == 0 && o.col_chunks != 0 &&
        (g.n_ct == 2 || g.n_ct == 4) && g.vec == (int)(16 / es) &&
        bd_bwd_has_signature(M, plan.n_cls[0], plan.n_cls[1], plan.n_cls[2], plan.n_cls[3], plan.absent, plan.share, (int)g.n_ct, false)) {
      chunks = (int)g.n_ct;
      g.n_ct = 1;
    }
    const int TY = kBlock >> g.log2_tx;
    // Sums over rows want many rows per block (fewer per-block partials for the second pass,
    // the LDS combine amortised), and measured best is a grid of one block per CU (256 on
    // MI355X): 8192 x 8192 runs 381 us at 256 rows per block, 399 us at 128, 434 us at 32.
    // The recompute kernels carry the op's arithmetic and want two blocks per CU to hide it
    // (same problem: 314 us at 128 rows per block, 478 us at 256).
    // So do the kernels that read the gradient table at run time (8192 x 8192 branchy5 forced onto
    // them: 419 us at 128 rows per block, 631 us at 256).
    const bool class_kernel = !rop && o.runtime_table == 0 && g.vec == (int)(16 / es) &&
                              bd_bwd_has_signature(M, plan.n_cls[0], plan.n_cls[1], plan.n_cls[2], plan.n_cls[3], plan.absent,
                                                   plan.share, 1, !uniform_stride);
    // A class kernel that streams many planes per row step is the exception (HM-LSTM update stored
    // [batch x hidden], 2 adjoints + 20 planes: 8192 x 4096 runs 733 us at two blocks per CU, 995 us at
    // one; with its 10 distinct planes, 509 us and 457 us).
    int planes_read = M;
    for (size_t e = 0; e < order.size(); ++e)
      for (int i = 0; i < M; ++i)
        planes_read += v[M + i * ND + order[e]].p != nullptr && !(e < 16 && ((plan.share >> (4 * e)) & 15u));
    const bool one_per_cu = class_kernel && planes_read < 16;
    // Small problems want about one block per CU whatever the kernel (per-block set-up and the final
    // combine weigh more than overlap): [512 x 2048] HM-LSTM, 1024 tiles of one row step, runs 23 us at
    // 4 row steps per block, 26 us at 2, 29 us at 8; [256 x 1024] 11-13 us at 1 or 2, 19 us at 8.
    const int64_t tiles = ceil_div(s2.R, TY) * g.n_ct * s2.O;  // row steps x column chunks of the whole problem
    int64_t steps_rowwise;
    if (one_per_cu) {
      steps_rowwise = std::min<int64_t>(512 / TY, tiles / 256);  // (fp64 8192 x 8192 branchy5: 512 steps, one block per CU, 700 us; 256 steps, two per CU, 747 us)
    } else {
      steps_rowwise = tiles / 512;
      if (steps_rowwise < 8) steps_rowwise = std::min<int64_t>(8, tiles / 256);
      steps_rowwise = std::min<int64_t>(128 / TY, steps_rowwise);
    }
    steps_rowwise = std::max<int64_t>(1, steps_rowwise);
    int steps = o.bwd_row_steps > 0 ? o.bwd_row_steps : (any_rowwise ? (int)steps_rowwise : auto_steps(s2.R, g, 4));
    if (class_kernel && !any_rowwise && o.bwd_row_steps == 0) steps = 1;  // signature kernels without row sums have no row loop
    if (rop) {
      uint64_t pattern = 0;  // 3 bits per differentiable argument: class + 1
      for (int j = 0; j < ND; ++j) pattern |= (uint64_t)(cls[j] + 1) << (3 * j);
      auto transposed = [](uint64_t q) {  // rows-only and columns-only swapped
        uint64_t t = 0;
        for (int j = 0; j < 20; ++j) {
          uint64_t cl = (q >> (3 * j)) & 7u;
          cl = cl == kGradRowSum + 1 ? kGradColSum + 1 : cl == kGradColSum + 1 ? kGradRowSum + 1 : cl;
          t |= cl << (3 * j);
        }
        return t;
      };
      plan.fixed_pattern = o.runtime_table != 0 ? 0 : pattern == rop->recompute_pattern() ? 1
                           : pattern == transposed(rop->recompute_pattern()) ? 2 : 0;
      // the fixed-pattern kernels take each argument's broadcast form from its gradient's class:
      // the argument's own strides must say the same (an expanded stride-0 view would not)
      for (int j = 0, jd = 0; j < NA && plan.fixed_pattern; ++j) {
        if ((rop->nondiff >> j) & 1u) continue;
        const TView tv = tview(c, a0 + j, v[a0 + j].p);
        const bool rows_fixed = cls[jd] == kGradColSum || cls[jd] == kGradAllSum;
        const bool cols_fixed = cls[jd] == kGradRowSum || cls[jd] == kGradAllSum;
        if ((s2.R > 1 && (tv.sr == 0) != rows_fixed) || (s2.C > 1 && (tv.sc == 0) != cols_fixed)) plan.fixed_pattern = 0;
        ++jd;
      }
      if (ragged && plan.fixed_pattern == 2) plan.fixed_pattern = 0;  // the unaligned form exists for the op's own pattern and the run-time one
      if (plan.fixed_pattern && !any_rowwise) {
        if (o.bwd_row_steps > 1) plan.fixed_pattern = 0;  // an explicit rows-per-block override needs the looping kernel
        else steps = 1;                                  // that kernel has no row loop
      }
    }
    // rows wider than a wavefront park one accumulator per wavefront and row in LDS
    const int wpr = g.log2_tx > 6 ? (1 << (g.log2_tx - 6)) : 1;
    if (g.log2_tx > 6 && n_rowsum > 0) {
      const int64_t max_rows = (int64_t)(kLdsBudget * 2 / 3) / ((int64_t)n_rowsum * wpr * as);
      steps = (int)std::max<int64_t>(1, std::min<int64_t>(steps, max_rows / TY));
    }
    if (!tile_rows(s2.R, steps, g)) return BCAST_ERR_LAUNCH_FAILED;
    if (g.n_ct * g.n_rt > 0x7fffffffLL / s2.O) return BCAST_ERR_LAUNCH_FAILED;
    plan.grid = dim3((unsigned)(s2.O * g.n_ct * g.n_rt), 1, 1);
    const int rows_pb = TY * g.steps;

    // Full-shape gradients are written with the nontemporal hint when there are so many bytes of them that
    // keeping them in the caches only displaces what the launch still has to read (256 MiB and more), or when
    // the planes the call reads are so few that the whole step lives in the memory-side cache anyway (see the
    // forward launch); in between plain stores measured faster.
    int n_fullgrads = 0, n_planes_read = M;
    for (int j = 0; j < ND; ++j) n_fullgrads += (cls[j] == kGradFull);
    for (int k = 0; k < M * ND; ++k) n_planes_read += (v[M + k].p != nullptr);
    const int64_t plane_bytes = s2.O * s2.R * s2.C * (int64_t)es;
    const bool nt_wanted = o.bwd_nt_min_mib >= 0 ? n_fullgrads * plane_bytes >= ((int64_t)o.bwd_nt_min_mib << 20)
                                                 : n_fullgrads * plane_bytes >= kNtGradientBytes || n_planes_read * plane_bytes <= kSmallStepBytes;
    const int32_t nt_gradients = ((o.nontemporal_stores >> 1) & 1) && n_fullgrads > 0 && nt_wanted;
    // split the gradients over launches so that each launch's LDS accumulators fit
    size_t ws = 0;
    plan.p2.n_jobs = 0;
    int64_t p2_blocks = 0;
    BwdTiledParams cur{};
    auto reset = [&](BwdTiledParams &p) {
      p = BwdTiledParams{};
      p.R = s2.R;
      p.C = s2.C;
      p.log2_tx = g.log2_tx;
      p.steps = g.steps;
      p.nt_store = nt_gradients;
      p.reverse = o.reverse_tiles;
      p.interleave = o.interleave_rows;
      p.xcd_remap = o.xcd_order != 0 && (s2.O * g.n_ct * g.n_rt) % 8 == 0;
      p.col_chunks = chunks;
      p.uniform_stride = uniform_stride;
      p.ragged = ragged;
      p.M = M;
      p.n_ct = g.n_ct;
      p.n_rt = g.n_rt;
      p.row_stride = bwd_sr;
      p.O = s2.O;
      p.tiles_per_slice = g.n_ct * g.n_rt;
      p.outer_stride = bwd_so;
      for (int i = 0; i < M; ++i) p.adj[i] = sview(c, i, v[i].p);
    };
    auto lds_need = [&](const BwdTiledParams &p, size_t &row_off, size_t &col_off, size_t &all_off) {
      size_t o = 0;
      row_off = o;
      if (g.log2_tx > 6) o += align16((size_t)p.n_row_slots * rows_pb * wpr * as);
      col_off = o;
      o += align16((size_t)p.n_col_slots * kBlock * g.vec * as);
      all_off = o;
      o += align16((size_t)p.n_all_slots * kBlock * as);
      return o;
    };
    auto flush = [&]() {
      if (cur.n_entries == 0) return;
      size_t ro, co, ao;
      const size_t total = lds_need(cur, ro, co, ao);
      cur.lds_row_off = (uint32_t)ro;
      cur.lds_col_off = (uint32_t)co;
      cur.lds_all_off = (uint32_t)ao;
      plan.main.push_back(cur);
      plan.main_lds.push_back(std::max<size_t>(total, (size_t)o.bwd_lds_kib * 1024));
    };
    reset(cur);
    for (int j : order) {
      BwdTiledParams trial = cur;
      trial.n_row_slots += (cls[j] == kGradRowSum);
      trial.n_col_slots += (cls[j] == kGradColSum);
      trial.n_all_slots += (cls[j] == kGradAllSum);
      size_t ro, co, ao;
      if (cur.n_entries > 0 && lds_need(trial, ro, co, ao) > kLdsBudget) {
        flush();
        reset(cur);
      }
      BwdEntry &en = cur.e[cur.n_entries++];
      for (int i = 0; i < M; ++i) en.P[i] = sview(c, M + i * ND + j, v[M + i * ND + j].p);
      en.g = tview(c, g0 + j, v[g0 + j].p);
      en.cls = cls[j];
      en.ws_off = 0;
      en.direct = 1;
      en.outer_sum = outer_sum[j];
      // the second pass's view of this gradient's partial sums (layouts: see Pass2Job); a gradient that
      // keeps the outer dim has O times the outputs, one summed over it O times the partials per output
      const int64_t O = s2.O, tiles_ps = g.n_ct * g.n_rt;
      const bool kept = O > 1 && !outer_sum[j];
      Pass2Job job{};
      job.g = en.g.p;
      job.g_outer_stride = en.g.so;
      job.n_outer = kept ? O : 1;
      if (cls[j] == kGradRowSum) {
        en.slot = cur.n_row_slots++;
        en.direct = g.n_ct == 1 && !outer_sum[j];
        job.g_stride = en.g.sr;
        job.outer_major = 0;  // output (r, o) = r * O + o
        job.n_out = kept ? s2.R * O : s2.R;
        job.n_part = kept ? g.n_ct : g.n_ct * O;
        job.part_stride = 1;
        job.out_stride = job.n_part;
        job.kind = job.n_part <= 256 ? 0 : 1;
        job.n_blocks = job.kind == 0 ? ceil_div(job.n_out, kBlock / 64) : job.n_out;
      } else if (cls[j] == kGradColSum) {
        en.slot = cur.n_col_slots++;
        en.direct = g.n_rt == 1 && !outer_sum[j];
        job.g_stride = en.g.sc;
        job.outer_major = 1;  // output (o, c) = o * C + c
        job.n_out = kept ? O * s2.C : s2.C;
        job.n_part = kept ? g.n_rt : g.n_rt * O;
        job.part_stride = kept ? O * s2.C : s2.C;
        job.out_stride = 1;
        // many partials per output: 16 outputs per block, each summed by 16 groups of lanes
        job.kind = job.n_part <= 32 ? 2 : 3;
        job.n_blocks = ceil_div(job.n_out, job.kind == 2 ? 64 : 16);
      } else if (cls[j] == kGradAllSum) {
        en.slot = cur.n_all_slots++;
        en.direct = tiles_ps == 1 && !outer_sum[j];
        job.g_stride = 0;
        job.outer_major = 1;  // output o
        job.n_out = kept ? O : 1;
        job.n_part = kept ? tiles_ps : tiles_ps * O;
        job.part_stride = kept ? O : 1;
        job.out_stride = kept ? 1 : 0;
        job.kind = 1;
        job.n_blocks = job.n_out;
      }
      if (!en.direct) {
        en.ws_off = (int64_t)ws;
        job.ws_off = (int64_t)ws;
        job.first_block = p2_blocks;
        p2_blocks += job.n_blocks;
        ws += align16((size_t)job.n_out * job.n_part * as);
        plan.p2.job[plan.p2.n_jobs++] = job;
      }
    }
    flush();
    if (rop) {
      if (plan.main.size() > 1) return BCAST_ERR_UNSUPPORTED;
      RecomputeArgs &ra = plan.ra;
      for (int jd = 0; jd < BCAST_MAX_ARGS; ++jd) ra.entry_of[jd] = -1;
      for (size_t e = 0; e < order.size(); ++e) ra.entry_of[order[e]] = (int8_t)e;
      for (int j = 0; j < NA; ++j) {
        const TView tv = tview(c, a0 + j, v[a0 + j].p);
        ra.arg_p[j] = tv.p;
        ra.arg_sr[j] = tv.sr;
        ra.arg_so[j] = tv.so;
        if (tv.sr == 0) ra.row_invariant |= 1u << j;
        if (tv.sc == 0) ra.col_invariant |= 1u << j;
      }
    }
    plan.signature = !rop && plan.main.size() == 1 && o.runtime_table == 0 && (int)order.size() * M <= 64 &&
                     (any_rowwise || g.steps == 1) &&  // those kernels loop over rows only when they sum over rows
                     bd_bwd_has_signature(M, plan.n_cls[0], plan.n_cls[1], plan.n_cls[2], plan.n_cls[3], plan.absent, plan.share, chunks,
                                          !uniform_stride);
    if (p2_blocks > 0x7fffffffLL) return BCAST_ERR_LAUNCH_FAILED;
    plan.p2_blocks = p2_blocks;
    plan.ws_bytes = ws;
    plan.info.path = 1;
    plan.info.vec = g.vec;
    plan.info.tx = 1 << g.log2_tx;
    plan.info.ty = TY;
    plan.info.rows_per_block = rows_pb;
    plan.info.grid_x = g.n_ct;
    plan.info.grid_y = g.n_rt * s2.O;
    plan.info.n_launches = (int)plan.main.size() + (p2_blocks > 0 ? 1 : 0);
    plan.info.n_second_pass = plan.p2.n_jobs;
    // the class-specialised kernels exist for the widest vector only
    plan.info.specialized = plan.signature && ((dt == BCAST_F32 && g.vec == 4) || (dt == BCAST_F64 && g.vec == 2));
    plan.info.ragged = ragged;
    plan.info.uniform_stride = uniform_stride;
    plan.info.nontemporal_tiles = nt_gradients && plan.info.specialized && uniform_stride && chunks == 1 ? g.n_ct * g.n_rt * s2.O : 0;
  } else {
    size_t gen_ws = 0;  // partial sums of the reductions that are cut into chunks
    for (int j = 0; j < ND; ++j) {
      if (!v[g0 + j].p) continue;
      BwdGenericParams p{};
      p.nd = c.nd;
      p.M = M;
      p.E = c.E;
      for (int d = 0; d < BCAST_MAX_DIMS; ++d) p.shape[d] = d < c.nd ? c.shape[d] : 1;
      for (int i = 0; i < M; ++i) {
        p.adj[i] = gview(c, i, v[i].p);
        p.P[i] = gview(c, M + i * ND + j, v[M + i * ND + j].p);
      }
      p.g = gview(c, g0 + j, v[g0 + j].p);
      p.n_kept = 1;
      p.n_fibre = 1;
      bool reduce = false;
      for (int d = 0; d < c.nd; ++d) {
        p.reduced[d] = (p.g.s[d] == 0);
        reduce |= p.reduced[d] != 0;
        (p.reduced[d] ? p.n_fibre : p.n_kept) *= c.shape[d];
      }
      int gv = !reduce && c.nd >= 1 ? (int)(std::max<int>(o.max_vector_bytes, (int)es) / es) : 1;
      if (gv != (int)(16 / es) || c.shape[c.nd - 1] % gv != 0) gv = 1;
      for (int i = 0; i < M && gv > 1; ++i) {
        if (!generic_vector_ok(c, i, v[i].p, gv, es, true)) gv = 1;
        const size_t tp = M + i * ND + j;
        if (gv > 1 && v[tp].p && !generic_vector_ok(c, tp, v[tp].p, gv, es, false)) gv = 1;
      }
      if (gv > 1 && !generic_vector_ok(c, g0 + j, v[g0 + j].p, gv, es, false)) gv = 1;
      p.vec = gv;
      p.splits = 1;
      int64_t blocks = ceil_div(c.E / gv, kBlock);
      if (reduce) {
        // enough blocks to fill the chip: a fibre is cut into chunks (at least 1024 terms each where
        // the lanes walk it, 64 where they lie along the gradient's elements)
        p.lanes_along_kept = c.nd >= 1 && !p.reduced[c.nd - 1];
        const int64_t groups = p.lanes_along_kept ? ceil_div(p.n_kept, 64) : p.n_kept;
        const int64_t min_chunk = p.lanes_along_kept ? 64 : 1024;
        int64_t splits = std::min<int64_t>(ceil_div(2048, groups), std::max<int64_t>(1, p.n_fibre / min_chunk));
        splits = std::max<int64_t>(1, std::min<int64_t>(splits, 4096));
        p.chunk = ceil_div(p.n_fibre, splits);
        splits = ceil_div(p.n_fibre, p.chunk);  // no empty chunk
        p.splits = (int32_t)splits;
        blocks = groups * splits;
        if (splits > 1) {
          p.ws_off = (int64_t)gen_ws;
          gen_ws += align16((size_t)p.n_kept * splits * as);
        }
      }
      if (blocks > 0x7fffffffLL) return BCAST_ERR_LAUNCH_FAILED;
      plan.generic.emplace_back(reduce ? 1 : 0, p);
      plan.generic_blocks.push_back(blocks);
      if (reduce && p.splits > 1) {
        plan.generic.emplace_back(2, p);
        plan.generic_blocks.push_back(ceil_div(p.n_kept, kBlock));
      }
    }
    plan.ws_bytes = gen_ws;
    plan.info.path = 2;
    plan.info.vec = 1;
    plan.info.tx = kBlock;
    plan.info.ty = 1;
    plan.info.rows_per_block = 1;
    plan.info.grid_x = plan.generic_blocks.empty() ? 0 : plan.generic_blocks[0];
    plan.info.grid_y = 1;
    plan.info.n_launches = (int)plan.generic.size();
  }
  return BCAST_OK;
}

}  // namespace

// ---- the C ABI ---------------------------------------------------------------------------------------
extern "C" {

int bcast_op_count(void) { return kNumOps; }

const char *bcast_op_name(int32_t op_id) { return (op_id >= 0 && op_id < kNumOps) ? kOps[op_id].name : nullptr; }

int bcast_op_lookup(const char *name, int32_t *op_id) {
  if (name == nullptr || op_id == nullptr) return BCAST_ERR_NULL_POINTER;
  for (int k = 0; k < kNumOps; ++k)
    if (std::strcmp(kOps[k].name, name) == 0) {
      *op_id = k;
      return BCAST_OK;
    }
  return BCAST_ERR_INVALID_OP;
}

int bcast_op_info(int32_t op_id, int32_t *n_args, int32_t *n_outputs, uint32_t *nondiff_mask,
                  int32_t *n_branches) {
  if (op_id < 0 || op_id >= kNumOps) return BCAST_ERR_INVALID_OP;
  if (n_args) *n_args = kOps[op_id].n_args;
  if (n_outputs) *n_outputs = kOps[op_id].n_out;
  if (nondiff_mask) *nondiff_mask = kOps[op_id].nondiff;
  if (n_branches) *n_branches = kOps[op_id].n_branches;
  return BCAST_OK;
}

int bcast_op_plane_alias(int32_t op_id, int32_t *alias) {
  if (op_id < 0 || op_id >= kNumOps) return BCAST_ERR_INVALID_OP;
  if (alias == nullptr) return BCAST_ERR_NULL_POINTER;
  const OpDesc &op = kOps[op_id];
  const int n = op.n_out * (op.n_args - __builtin_popcount(op.nondiff));
  for (int k = 0; k < n; ++k) alias[k] = op.alias ? op.alias[k] : k;
  return BCAST_OK;
}

void bcast_dual_options_default(bcast_dual_options *opt) {
  if (opt != nullptr) default_options(*opt);
}

int bcast_dual_forward_plan(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                            int32_t n_out, const bcast_tensor *outs, const bcast_tensor *partials,
                            const uint8_t *branch_id, bcast_plan_info *info, const bcast_dual_options *opt) {
  if (info == nullptr) return BCAST_ERR_NULL_POINTER;
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  FwdPlan plan;
  const int rc = plan_forward(op_id, (int)dt, n_args, args, n_out, outs, partials, branch_id, o, plan);
  if (rc == BCAST_OK) *info = plan.info;
  return rc;
}

int bcast_dual_forward(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                       int32_t n_out, const bcast_tensor *outs, const bcast_tensor *partials,
                       uint8_t *branch_id, void *stream, const bcast_dual_options *opt) {
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  FwdPlan plan;
  const int rc = plan_forward(op_id, (int)dt, n_args, args, n_out, outs, partials, branch_id, o, plan);
  if (rc != BCAST_OK) return rc;
  if (plan.info.path == 0) return BCAST_OK;
  const Launch L = on_stream(stream, &o);
  hipError_t err = plan.tiled ? kOps[op_id].tiled((int)dt, plan.info.vec, plan.tp, plan.grid, L)
                              : kOps[op_id].generic((int)dt, plan.gp, plan.grid, L);
  return launch_status(err);
}

size_t bcast_dual_backward_workspace(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                                     const bcast_tensor *partials, int32_t n_grads,
                                     const bcast_tensor *grads, const bcast_dual_options *opt) {
  Opt o;
  if (resolve_options(opt, o) != BCAST_OK) return 0;
  BwdPlan plan;
  if (plan_backward((int)dt, n_out, adjoints, partials, n_grads, grads, o, plan) != BCAST_OK) return 0;
  return plan.ws_bytes;
}

int bcast_dual_backward_plan(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                             const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                             bcast_plan_info *info, const bcast_dual_options *opt) {
  if (info == nullptr) return BCAST_ERR_NULL_POINTER;
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  BwdPlan plan;
  const int rc = plan_backward((int)dt, n_out, adjoints, partials, n_grads, grads, o, plan);
  if (rc == BCAST_OK) *info = plan.info;
  return rc;
}

// workspace checks shared by the launching calls
static int check_workspace(const BwdPlan &plan, const void *workspace, size_t workspace_bytes) {
  if (plan.ws_bytes == 0) return BCAST_OK;
  if (workspace == nullptr) return BCAST_ERR_NULL_POINTER;
  if (workspace_bytes < plan.ws_bytes) return BCAST_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return BCAST_ERR_MISALIGNED;
  return BCAST_OK;
}

// enqueue what plan_backward laid out (cached planes; tiled or generic)
static int run_backward(int dt, BwdPlan &plan, void *workspace, void *stream, const Opt &o) {
  const Launch timed = on_stream(stream, &o), plain = on_stream(stream);
  if (plan.tiled) {
    for (size_t k = 0; k < plan.main.size(); ++k) {
      plan.main[k].ws = static_cast<unsigned char *>(workspace);
      if (launch_status(bd_bwd_tiled(dt, plan.vec, plan.signature, plan.n_cls[0], plan.n_cls[1], plan.n_cls[2], plan.n_cls[3],
                                     plan.absent, plan.share, plan.main[k], plan.grid, plan.main_lds[k], k == 0 ? timed : plain)) != BCAST_OK)
        return BCAST_ERR_LAUNCH_FAILED;
    }
    if (plan.p2_blocks > 0) {
      plan.p2.ws = static_cast<unsigned char *>(workspace);
      if (launch_status(bd_bwd_pass2(dt, plan.p2, plan.p2_blocks, plain)) != BCAST_OK) return BCAST_ERR_LAUNCH_FAILED;
    }
  } else {
    for (size_t k = 0; k < plan.generic.size(); ++k) {
      plan.generic[k].second.ws = static_cast<unsigned char *>(workspace);
      if (launch_status(bd_bwd_generic(dt, plan.generic[k].first, plan.generic[k].second, plan.generic_blocks[k],
                                       k == 0 ? timed : plain)) != BCAST_OK)
        return BCAST_ERR_LAUNCH_FAILED;
    }
  }
  return BCAST_OK;
}

int bcast_dual_backward(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                        const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                        void *workspace, size_t workspace_bytes, void *stream, const bcast_dual_options *opt) {
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  BwdPlan plan;
  const int rc = plan_backward((int)dt, n_out, adjoints, partials, n_grads, grads, o, plan);
  if (rc != BCAST_OK) return rc;
  if (plan.info.path == 0) return BCAST_OK;
  if (int wrc = check_workspace(plan, workspace, workspace_bytes)) return wrc;
  return run_backward((int)dt, plan, workspace, stream, o);
}

// ---- the entry point that allocates nothing ---------------------------------------------------------
// Scratch memory of the second reduction pass as part of the device image: one copy per GPU.  On the
// host this name only stands for the symbol; the memory's address on a GPU comes from
// hipGetSymbolAddress, once per device, and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[BCAST_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];  // per device, written once (every writer stores the same address)

int scratch_of_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    std::fprintf(stderr, "bcast_dual: no current device for the static scratch array: %s\n", hipGetErrorString(e));
    return BCAST_ERR_LAUNCH_FAILED;
  }
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      std::fprintf(stderr, "bcast_dual: hipGetSymbolAddress of the static scratch array failed on device %d: %s\n", dev,
                   hipGetErrorString(e));
      return BCAST_ERR_LAUNCH_FAILED;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return BCAST_OK;
}
}  // namespace

int bcast_dual_backward_noalloc(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                                const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                                void *stream, const bcast_dual_options *opt) {
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  BwdPlan plan;
  const int rc = plan_backward((int)dt, n_out, adjoints, partials, n_grads, grads, o, plan);
  if (rc != BCAST_OK) return rc;
  if (plan.info.path == 0) return BCAST_OK;
  if (plan.ws_bytes > (size_t)BCAST_NOALLOC_SCRATCH_BYTES) return BCAST_ERR_WORKSPACE_TOO_SMALL;
  void *ws = nullptr;
  if (plan.ws_bytes > 0)
    if (int src = scratch_of_current_device(&ws)) return src;
  return run_backward((int)dt, plan, ws, stream, o);
}

static int recompute_plan(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args, int32_t n_out,
                          const bcast_tensor *adjoints, int32_t n_grads, const bcast_tensor *grads, const Opt &o, BwdPlan &plan) {
  if (op_id < 0 || op_id >= kNumOps) return BCAST_ERR_INVALID_OP;
  const OpDesc &op = kOps[op_id];
  if (n_args != op.n_args || n_out != op.n_out || n_grads != op.n_args - __builtin_popcount(op.nondiff))
    return BCAST_ERR_BAD_ARG_COUNT;
  if (op.recompute == nullptr) return BCAST_ERR_UNSUPPORTED;
  return plan_backward((int)dt, n_out, adjoints, nullptr, n_grads, grads, o, plan, &op, args);
}

size_t bcast_dual_backward_recompute_workspace(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                               int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                               const bcast_tensor *grads, const bcast_dual_options *opt) {
  Opt o;
  if (resolve_options(opt, o) != BCAST_OK) return 0;
  BwdPlan plan;
  if (recompute_plan(op_id, dt, n_args, args, n_out, adjoints, n_grads, grads, o, plan) != BCAST_OK) return 0;
  return plan.ws_bytes;
}

int bcast_dual_backward_recompute_plan(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                       int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                       const bcast_tensor *grads, bcast_plan_info *info, const bcast_dual_options *opt) {
  if (info == nullptr) return BCAST_ERR_NULL_POINTER;
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  BwdPlan plan;
  const int rc = recompute_plan(op_id, dt, n_args, args, n_out, adjoints, n_grads, grads, o, plan);
  if (rc == BCAST_OK) {
    *info = plan.info;
    info->specialized = plan.info.path == 1 && plan.fixed_pattern ? 1 : 0;
  }
  return rc;
}

int bcast_dual_backward_recompute(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                  int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                  const bcast_tensor *grads, void *workspace, size_t workspace_bytes, void *stream,
                                  const bcast_dual_options *opt) {
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  BwdPlan plan;
  const int rc = recompute_plan(op_id, dt, n_args, args, n_out, adjoints, n_grads, grads, o, plan);
  if (rc != BCAST_OK) return rc;
  if (plan.info.path == 0 || plan.main.empty()) return BCAST_OK;
  if (int wrc = check_workspace(plan, workspace, workspace_bytes)) return wrc;
  plan.main[0].ws = static_cast<unsigned char *>(workspace);
  if (launch_status(kOps[op_id].recompute((int)dt, plan.vec, plan.fixed_pattern, plan.main[0], plan.ra, plan.grid,
                                          plan.main_lds[0], on_stream(stream, &o))) != BCAST_OK)
    return BCAST_ERR_LAUNCH_FAILED;
  if (plan.p2_blocks > 0) {
    plan.p2.ws = static_cast<unsigned char *>(workspace);
    if (launch_status(bd_bwd_pass2((int)dt, plan.p2, plan.p2_blocks, on_stream(stream))) != BCAST_OK) return BCAST_ERR_LAUNCH_FAILED;
  }
  return BCAST_OK;
}

const char *bcast_status_string(int status) {
  switch (status) {
    case BCAST_OK: return "ok";
    case BCAST_ERR_INVALID_OP: return "invalid op";
    case BCAST_ERR_BAD_ARG_COUNT: return "wrong number of arguments, outputs or gradients";
    case BCAST_ERR_NULL_POINTER: return "null pointer";
    case BCAST_ERR_RANK_TOO_HIGH: return "rank exceeds BCAST_MAX_DIMS";
    case BCAST_ERR_SHAPE_MISMATCH: return "argument shapes do not broadcast";
    case BCAST_ERR_OUTPUT_SHAPE_MISMATCH: return "output, partial, adjoint or gradient view has the wrong shape";
    case BCAST_ERR_BAD_DTYPE: return "unknown dtype";
    case BCAST_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case BCAST_ERR_LAUNCH_FAILED: return "kernel launch failed";
    case BCAST_ERR_BAD_STRIDE: return "negative stride or self-overlapping written view";
    case BCAST_ERR_MISALIGNED: return "pointer not aligned";
    case BCAST_ERR_UNSUPPORTED: return "layout or op not supported by this entry point";
    case BCAST_ERR_BAD_OPTION: return "an option is outside its range, or the options struct has the wrong size";
    default: return "unknown status";
  }
}

size_t bcast_dual_slab_layout(size_t plane_bytes, int32_t n_planes, size_t *offsets) {
  if (n_planes <= 0) return 0;
  // HBM channels interleave at 4 KiB: planes whose starts differ by a multiple of a large
  // power of two put the same element of every plane on the same channel.  One extra 4 KiB
  // page per plane staggers them.  Small planes are only aligned.
  const size_t page = 4096;
  const size_t rounded = (plane_bytes + page - 1) / page * page;
  const size_t stride = plane_bytes >= (size_t)1 << 20 ? rounded + page : (plane_bytes + 255) / 256 * 256;
  if (offsets)
    for (int32_t k = 0; k < n_planes; ++k) offsets[k] = (size_t)k * stride;
  return (size_t)n_planes * stride;
}

int bcast_dual_stream_probe(int32_t n_in, const void *const *in, const int64_t *in_chunk_stride, int32_t n_out,
                            void *const *out, const int64_t *out_chunk_stride, int64_t n_chunks, void *stream,
                            const bcast_dual_options *opt) {
  Opt o;
  if (int rc = resolve_options(opt, o)) return rc;
  if (n_in < 0 || n_in > 32 || n_out < 0 || n_out > 32 || n_in + n_out == 0) return BCAST_ERR_BAD_ARG_COUNT;
  if ((n_in && (!in || !in_chunk_stride)) || (n_out && (!out || !out_chunk_stride))) return BCAST_ERR_NULL_POINTER;
  if (n_chunks < 0 || n_chunks > 0x7fffffffLL) return BCAST_ERR_LAUNCH_FAILED;
  for (int k = 0; k < n_in; ++k) {
    if (!in[k]) return BCAST_ERR_NULL_POINTER;
    if (reinterpret_cast<uintptr_t>(in[k]) % 16 || in_chunk_stride[k] % 4 || in_chunk_stride[k] < 0) return BCAST_ERR_MISALIGNED;
  }
  for (int k = 0; k < n_out; ++k) {
    if (!out[k]) return BCAST_ERR_NULL_POINTER;
    if (reinterpret_cast<uintptr_t>(out[k]) % 16 || out_chunk_stride[k] % 4 || out_chunk_stride[k] < 1024) return BCAST_ERR_MISALIGNED;
  }
  if (n_chunks == 0) return BCAST_OK;
  return launch_status(bd_stream_probe(n_in, in, in_chunk_stride, n_out, out, out_chunk_stride, n_chunks, o.probe_nt_loads != 0,
                                       o.reverse_tiles == 1, (size_t)o.probe_lds_kib * 1024, on_stream(stream, &o)));
}

}  // extern "C"
