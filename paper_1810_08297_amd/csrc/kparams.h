// Kernel argument blocks shared by the host planner and the HIP kernels.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "bcast_dual.h"

namespace bd {

constexpr int kBlock = 256;  // threads per block of every tiled kernel (4 wavefronts)

// A 2-D view used by the tiled kernels: element (r, c) lives at p + r*sr + c*sc.
// For tensors read or written with vector instructions sc is 0 or 1.  A lane's address is a
// 64-bit part common to its block (base pointer + first row of the block's row step * sr, in
// scalar registers) plus a 32-bit byte offset of its own (its row within the step and its
// column): views may be of any size, only the TY rows of one step must span less than 4 GiB.
// In the usual case every view that varies along both rows and columns shares ONE row stride
// (row_stride of the parameter block): both parts are then computed once per row step and
// serve every plane.  Otherwise (uniform_stride == 0: arguments or gradients that are slices
// of wider buffers) a second instantiation of the kernels forms them per view from its own sr.
// A problem of three merged dims is a batch of O such 2-D problems (slices): the block grid is
// laid out O times, a block takes its slice from its index, and element (o, r, c) of a view lives
// at p + o*so + r*sr + c*sc.  Views that vary along all dims normally share so as well as sr.
struct TView {
  void *p;
  int64_t sr;
  int64_t sc;
  int64_t so;
};
// A view the backward kernels stream with vector loads (an adjoint, a plane): its column stride is 1.
struct SView {
  void *p;
  int64_t sr;
  int64_t so;
};

struct FwdTiledParams {
  int64_t R, C;        // rows, columns of the merged 2-D problem
  int32_t log2_tx;     // lanes along the columns = 1 << log2_tx; rows per step = 256 >> log2_tx
  int32_t lds_bytes;   // dynamic LDS requested at launch; the kernel does not touch it, it limits the blocks per CU
  uint32_t nt_tiles;   // tiles [0, nt_tiles) of the walk are written with the nontemporal hint, the rest plainly
  int32_t has_partials;
  int32_t xcd_remap;   // 1: consecutive tiles go to one XCD (block b of a grid of 8 n serves tile (b % 8) n + b / 8)
  int64_t n_ct;        // column tiles; block b of a slice serves column tile b % n_ct of row tile b / n_ct
  int64_t row_stride;  // elements between rows of every full-shape view (0 when R == 1)
  int64_t O;           // slices (extent of the outer dim of a 3-D problem; 1 otherwise)
  int64_t tiles_per_slice;  // blocks per slice; block B of the grid serves block B % tiles_per_slice of slice B / tiles_per_slice
  int64_t outer_stride;     // elements between slices of every full-shape view (0 when O == 1)
  uint32_t row_invariant;  // bit j: argument j does not vary along the rows
  uint32_t col_invariant;  // bit j: argument j does not vary along the columns
  // pointers are kept apart from the rarely used strides so that a few wide scalar loads
  // fetch them and nothing else occupies scalar registers
  const void *arg_p[BCAST_MAX_ARGS];
  void *out_p[BCAST_MAX_OUTS];
  void *part_p[BCAST_MAX_PLANES];  // nullptr: plane not stored
  uint8_t *branch_p;               // nullptr: not requested
  int64_t branch_sr, branch_sc;
  int64_t arg_sr[BCAST_MAX_ARGS];  // row stride of every argument, in elements
  // When the full-shape views do not share one row stride (uniform_stride == 0) every view is
  // addressed with its own.
  int32_t uniform_stride;
  // 1: rows of a length or at a start that is not a multiple of the vector; the kernel takes
  // unaligned vectors and the row's last columns singly (only with uniform_stride, C >= the vector)
  int32_t ragged;
  int64_t out_sr[BCAST_MAX_OUTS];
  int64_t part_sr[BCAST_MAX_PLANES];
  // outer strides (3-D problems): of every argument, always used; of outputs, planes and branch ids, used
  // like the row strides above when the views do not share one
  int64_t arg_so[BCAST_MAX_ARGS];
  int64_t out_so[BCAST_MAX_OUTS];
  int64_t part_so[BCAST_MAX_PLANES];
  int64_t branch_so;
};

// A strided view of up to BCAST_MAX_DIMS merged dims for the generic kernels.
struct GView {
  void *p;
  int64_t s[BCAST_MAX_DIMS];
};

struct FwdGenericParams {
  int32_t nd;
  int32_t vec;  // elements per lane along the innermost dim (1, or the 16-byte vector where every view allows it)
  int64_t shape[BCAST_MAX_DIMS];
  int64_t E;
  GView arg[BCAST_MAX_ARGS];
  GView out[BCAST_MAX_OUTS];
  GView part[BCAST_MAX_PLANES];
  GView branch;
};

// ---- backward ------------------------------------------------------------------------
enum GradClass : int32_t {
  kGradSkip = -1,
  kGradFull = 0,    // gradient has the output's shape: elementwise product (Table 1)
  kGradRowSum = 1,  // argument varied along rows only: sum over columns
  kGradColSum = 2,  // argument varied along columns only: sum over rows
  kGradAllSum = 3,  // scalar argument: sum over everything
};

struct BwdEntry {
  SView P[BCAST_MAX_OUTS];  // planes d Y_i / d X_j for this j; p == nullptr: zeros
  TView g;                  // gradient view (sr/sc are 0 on reduced dims)
  int32_t cls;
  int32_t slot;             // index among the entries of the same class in this launch
  int64_t ws_off;           // byte offset of this entry's partial sums in the workspace
  int32_t direct;           // 1: this launch writes the final gradient (no second pass)
  int32_t outer_sum;        // 1: the gradient is also summed over the slices of a 3-D problem (always through the second pass)
};

struct BwdTiledParams {
  int64_t R, C;
  int32_t log2_tx, steps, nt_store, M;
  int32_t n_entries;
  int32_t reverse;  // 1: blocks walk the tiles from the last to the first; 2: the same in groups of eight blocks, each keeping its place in its group
  int32_t xcd_remap;   // as in FwdTiledParams
  int32_t uniform_stride;  // 0: the full-shape views have row strides of their own (TView::sr of each)
  int32_t col_chunks;  // column chunks of TX * VEC columns a block covers per row step (0 or 1: one)
  int32_t interleave;  // 1: row tile rt takes row steps rt, rt + n_rt, rt + 2 n_rt, ... instead of a contiguous run
  int32_t ragged;      // as in FwdTiledParams (the run-time-table and recompute kernels only)
  int32_t n_row_slots, n_col_slots, n_all_slots;
  uint32_t lds_row_off, lds_col_off, lds_all_off;  // byte offsets into dynamic LDS
  int64_t n_ct, n_rt;  // column tiles, row tiles of one slice; block b of a slice = rt * n_ct + ct
  int64_t row_stride;  // elements between rows of every full-shape view (0 when R == 1)
  int64_t O, tiles_per_slice, outer_stride;  // as in FwdTiledParams
  unsigned char *ws;
  SView adj[BCAST_MAX_OUTS];
  BwdEntry e[BCAST_MAX_ARGS];
};

// The arguments of the broadcast, for the kernel that evaluates the dual numbers again in
// the reverse pass instead of reading cached planes.
struct RecomputeArgs {
  uint32_t row_invariant, col_invariant;   // as in FwdTiledParams
  const void *arg_p[BCAST_MAX_ARGS];
  int64_t arg_sr[BCAST_MAX_ARGS];
  int64_t arg_so[BCAST_MAX_ARGS];
  int8_t entry_of[BCAST_MAX_ARGS];         // differentiable argument jd -> row of the gradient table, -1: skipped
};

// second pass: one job per gradient that needs it
// Workspace layouts of the main pass (accumulator elements; O slices, o the block's slice):
//   row sums  [(r * O + o) * n_ct + ct]      column sums  [(rt * O + o) * C + c]      full sums  [b * O + o]
// (b: block within its slice).  A gradient that keeps the outer dim has O times the outputs, one that sums over
// it O times the partials per output; with O = 1 these are the layouts of a 2-D problem.
struct Pass2Job {
  void *g;              // final gradient
  int64_t g_stride;     // elements between consecutive outputs of one slice
  int64_t g_outer_stride;  // elements between slices (outputs that keep the outer dim)
  int64_t n_outer;      // 1, or O when the outputs keep the outer dim: output index = (inner, slice) ...
  int32_t outer_major;  // ... as slice * n_inner + inner (1) or inner * n_outer + slice (0)
  int32_t pad0;
  int64_t n_out;        // outputs of this job (over all slices)
  int64_t n_part;       // partial sums per output
  int64_t part_stride;  // in accumulator elements: between partials of one output
  int64_t out_stride;   // in accumulator elements: between outputs
  int64_t ws_off;       // bytes
  int64_t first_block;  // blocks [first_block, first_block + n_blocks) serve this job
  int64_t n_blocks;
  int32_t kind;         // 0: one wavefront per output, 1: one block per output, 2: 64 outputs x 4 groups per block,
                        // 3: 16 outputs x 16 groups per block
  int32_t pad;
};
struct Pass2Params {
  int32_t n_jobs;
  int32_t pad;
  unsigned char *ws;
  Pass2Job job[BCAST_MAX_ARGS];
};

struct BwdGenericParams {
  int32_t nd, M;
  int32_t vec, pad;  // as in FwdGenericParams (elementwise kernel only)
  int64_t shape[BCAST_MAX_DIMS];
  int64_t E;
  GView adj[BCAST_MAX_OUTS];
  GView P[BCAST_MAX_OUTS];
  GView g;
  // reduction geometry: kept dims enumerate gradient elements, reduced dims the fibre
  int32_t reduced[BCAST_MAX_DIMS];
  int64_t n_kept, n_fibre;
  // The fibre of every gradient element is cut into `splits` chunks of `chunk` terms, one block
  // each.  lanes_along_kept = 0: the innermost dim is reduced, a block serves one gradient element
  // and its lanes walk the fibre; 1: the innermost dim is kept, a block serves 64 consecutive
  // gradient elements (lanes along them: coalesced) with its four wavefronts interleaved over the
  // chunk.  With one chunk the block writes the gradient, otherwise its partial sum goes to
  // ws[element * splits + chunk] for the final kernel.
  int32_t splits, lanes_along_kept;
  int64_t chunk;
  int64_t ws_off;  // bytes
  unsigned char *ws;
};

}  // namespace bd
