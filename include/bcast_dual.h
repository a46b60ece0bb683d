/*
 * bcast_dual -- mixed-mode differentiation of a fused broadcast on one AMD
 * MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * Method: "Dynamic Automatic Differentiation of GPU Broadcast Kernels"
 * (arXiv 1810.08297).  A scalar function b : R^N -> R^M from the built-in op table
 * is broadcast over N array arguments (Sec. 2.1.1).  The forward call evaluates b on
 * multidimensional dual numbers, one perturbation per differentiable argument
 * (Sec. 2.2.1, the D operator of Sec. 2.2.2), in ONE kernel, data-dependent branches
 * included, and returns the M outputs together with the M x N_d planes
 * d Y_i / d X_j -- the diagonal of the broadcast Jacobian (Sec. 2.2.2).  The caller
 * keeps those planes until the reverse pass (Sec. 2.2.3); the backward call then
 * multiplies the upstream adjoints by them and sums over the dims along which each
 * argument was expanded (Table 1).
 *
 * Common rules
 *  - Every `data` pointer is a DEVICE pointer owned by the caller.  The library
 *    allocates no device memory, never synchronises, and enqueues work only on the
 *    `stream` argument (a hipStream_t; NULL = the default stream).
 *  - The library holds no mutable state: every call is a function of its arguments,
 *    and calls from different host threads need no locking.  (The one exception is stated
 *    where it applies: bcast_dual_backward_noalloc and its per-GPU scratch array.)
 *  - Views: `ndim` dims, extents `shape[d]`, strides `stride[d]` in ELEMENTS (may be
 *    any integer >= 0 that keeps the view inside its buffer; ignored where
 *    shape[d] == 1).  Dims an argument lacks are TRAILING size-1 dims, as in the
 *    paper's example where an n-vector pairs with the first dim of an n x m matrix
 *    (Sec. 2.1.1, Eq. 1).  A size-1 dim is virtually copied; it is never materialised.
 *  - All validation happens on the host before anything is launched; on any error
 *    nothing is written.  Return value: BCAST_OK (0) or a negative bcast_status.
 *  - Buffers written by a call must not overlap any other buffer of that call.
 *  - Zero-sized outputs: BCAST_OK, nothing is launched.
 *  - Results are bitwise reproducible run to run: no atomics, fixed reduction order.
 */
#ifndef BCAST_DUAL_H
#define BCAST_DUAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BCAST_MAX_DIMS 4
#define BCAST_MAX_ARGS 20
#define BCAST_MAX_OUTS 4
#define BCAST_MAX_PLANES 40 /* limit on M * N_d */

typedef enum { BCAST_F32 = 0, BCAST_F64 = 1 } bcast_dtype;

typedef enum {
  BCAST_OK = 0,
  BCAST_ERR_INVALID_OP = -1,
  BCAST_ERR_BAD_ARG_COUNT = -2,
  BCAST_ERR_NULL_POINTER = -3,
  BCAST_ERR_RANK_TOO_HIGH = -4,
  BCAST_ERR_SHAPE_MISMATCH = -5,        /* an argument dim is neither the unified extent nor 1 */
  BCAST_ERR_OUTPUT_SHAPE_MISMATCH = -6, /* an output / partial / adjoint / gradient view has the wrong shape */
  BCAST_ERR_BAD_DTYPE = -7,
  BCAST_ERR_WORKSPACE_TOO_SMALL = -8,
  BCAST_ERR_LAUNCH_FAILED = -9,
  BCAST_ERR_BAD_STRIDE = -10,           /* negative stride, or a written view that overlaps itself */
  BCAST_ERR_MISALIGNED = -11,           /* a data pointer is not aligned to its element size */
  BCAST_ERR_UNSUPPORTED = -12,          /* this entry point has no kernel for the op or the layout */
  BCAST_ERR_BAD_OPTION = -13            /* a field of bcast_dual_options is outside its documented range */
} bcast_status;

typedef struct {
  void *data;                    /* device pointer */
  int32_t ndim;                  /* 0 = scalar */
  int64_t shape[BCAST_MAX_DIMS];
  int64_t stride[BCAST_MAX_DIMS]; /* in elements */
} bcast_tensor;

/* How a call was (or would be) mapped onto the GPU; filled by the *_plan calls. */
typedef struct {
  int32_t path;     /* 0 nothing to do, 1 tiled kernels (the problem merges to two dims, or to three: then a batch
                       of two-dim slices), 2 generic strided kernels */
  int32_t vec;      /* elements per lane per memory instruction */
  int32_t ndim;     /* rank after dropping size-1 dims and merging mergeable dims */
  int64_t shape[BCAST_MAX_DIMS]; /* merged output extents, outermost first */
  int32_t tx, ty;   /* lanes along the contiguous dim / rows per block step */
  int32_t rows_per_block;
  int64_t grid_x, grid_y;
  int32_t n_launches; /* kernels this call enqueues */
  int32_t n_second_pass; /* gradients finished by the second reduction pass */
  int32_t specialized; /* backward: 1 if the main pass is a kernel compiled for this call's mix of
                          gradient classes, absent and shared planes; 0 = the kernels that read the
                          gradient table at run time.  forward: 0 */
  int32_t ragged;      /* 1: the rows do not fit the 16-byte vector (length, start or stride off its
                          boundary) and the kernels that take it unaligned, with the last columns of
                          every row singly, are used */
  int32_t uniform_stride; /* tiled path: 1 if every view the kernels stream row by row has the same row
                          stride (one address offset per lane then serves them all), 0 if each is addressed
                          with its own (slices of wider buffers, views that repeat one row) */
  int64_t nontemporal_tiles; /* forward, tiled path: how many tiles, counted from the start of the kernel's walk,
                          are written with the nontemporal hint (0: none; grid_x * grid_y: all; see
                          bcast_dual_options.fwd_keep_mib).  backward: the blocks of the main pass that write
                          full-shape gradients with the hint (0 or all; only the kernels compiled for a mix,
                          with one common row stride and one column chunk per block, have that form) */
} bcast_plan_info;

/* Per-call options.  Every entry point that plans or launches takes a `const bcast_dual_options *`
 * as its last argument; NULL means the defaults (the measured best on MI355X), which is what a
 * caller normally passes.  The library keeps no state between calls and none that two threads
 * could share: two calls with different options may run concurrently from different host threads.
 * The fields exist for launch-shape sweeps, for tests that force a particular kernel, and for
 * timing one launch; fill the struct with bcast_dual_options_default() first, then change fields.
 * A value outside its range makes the call return BCAST_ERR_BAD_OPTION before anything is launched.
 * A workspace query, a plan query and the call itself must be given the same options. */
typedef struct {
  uint32_t struct_size;     /* sizeof(bcast_dual_options) as the caller compiled it; any other value is refused */
  int32_t bwd_row_steps;    /* row steps per block of the tiled backward kernels: 0 (default) = automatic, else 1..512 */
  int32_t nontemporal_stores; /* bit 0: the forward kernel may write outputs and planes with the nontemporal hint
                               (see fwd_keep_mib), bit 1: the backward kernels may write full-shape gradients with it
                               (see bwd_nt_min_mib); default 3 = both */
  int32_t force_generic;    /* 1 = the generic strided kernels even where the tiled ones apply (testing); default 0 */
  int32_t max_vector_bytes; /* widest vector access per lane: 16 (default), 8 or 4 */
  int32_t runtime_table;    /* 1 = never a backward / recompute kernel compiled for the call's mix of gradient
                               classes, always the one that reads the gradient table at run time (testing); default 0 */
  int32_t reverse_tiles;    /* order in which the blocks of the tiled backward kernels take their tiles: 0 = first to
                               last; 1 = last to first, starting with the planes the forward kernel wrote last, which
                               the memory-side cache may still hold; 2 (default) = last to first in groups of eight
                               blocks, each block keeping its place within its group -- the hardware deals consecutive
                               blocks round-robin to the 8 XCDs, so a tile then stays on the XCD (its L2, its
                               address-translation cache) that wrote it in the forward kernel */
  int32_t interleave_rows;  /* rows of a backward block that takes several row steps: 1 (default) = every n-th row
                               step of the problem (the resident blocks sweep one contiguous band of each plane
                               together), 0 = one contiguous run of rows per block */
  int32_t xcd_order;        /* 1 = XCD-aware tile order: the hardware deals consecutive blocks round-robin to the
                               8 XCDs, and block b then serves tile (b % 8) * (blocks / 8) + b / 8, so that every
                               XCD gets one contiguous eighth of the tiles; 0 (default) = tile b.  Measured slower:
                               nothing is reused between blocks, and the eight bands sit a power of two apart */
  int32_t col_chunks;       /* 1 (default) = where a kernel was built for it, a backward block takes all 2 or 4
                               column chunks of a row, so that row sums of rows up to 4 x 1024 (fp64: 4 x 512)
                               elements finish in the main pass; 0 = one chunk per block */
  int32_t fwd_lds_kib;      /* KiB of (unused) dynamic LDS the forward kernel requests per block when it writes at
                               least 2.5 planes for every plane it reads, which limits the blocks resident on a CU
                               (160 KiB each): -1 (default) = automatic (48 = three blocks for fp32, 40 = four for
                               fp64), 0 = no limit; -1..64 */
  int32_t bwd_lds_kib;      /* the same for the main backward and recompute kernels, on top of what they need
                               (default 0: measured no gain); 0..64 */
  int32_t narrow_tiles;     /* 1 (default) = rows longer than 1024 elements may be tiled with 64 or 128 lanes per
                               row (4 or 2 rows per block step) where that pads the row less than 256 lanes */
  int32_t ragged_rows;      /* 1 (default) = rows whose length, start or stride is not a multiple of the 16-byte
                               vector are still read and written in such vectors, unaligned, with the last columns
                               of every row taken singly; 0 = the widest aligned access that fits (8 or 4 bytes) */
  int32_t probe_nt_loads;   /* bcast_dual_stream_probe: 1 (default) = nontemporal loads, 0 = plain */
  int32_t probe_lds_kib;    /* bcast_dual_stream_probe: unused dynamic LDS per block, as fwd_lds_kib (default 0) */
  int32_t fwd_keep_mib;     /* MiB of outputs and planes, counted from the end of what the forward kernel writes, that
                               it writes plainly so that they stay cached for a reverse pass that starts with them;
                               everything before is written with the nontemporal hint (streamed past the caches).
                               -1 (default) = automatic (a launch that writes up to 1 GiB: all of it; a larger one:
                               128); 0..1048576; a launch that writes no more than this is written plainly throughout */
  int32_t bwd_nt_min_mib;   /* MiB of full-shape gradients written by one backward call from which on they are written
                               with the nontemporal hint (bit 1 of nontemporal_stores permitting): -1 (default) =
                               automatic (256), 0 = always; 0..1048576 */
  /* Timing of one launch by the runtime itself: two hipEvent_t the caller created with timing enabled, both
   * or neither.  The main-pass kernel of the call (the forward kernel, the main backward or recompute kernel
   * -- the first one if the gradients need several launches, never the second reduction pass -- or the probe
   * kernel) stamps them with its own begin and end, so that hipEventElapsedTime(start, stop) is the kernel's
   * duration with no launch gap in it.  Not for a stream that is being captured into a graph. */
  void *start_event;
  void *stop_event;
} bcast_dual_options;

/* Fills *opt with the defaults (and struct_size). */
void bcast_dual_options_default(bcast_dual_options *opt);

/* ---- op table --------------------------------------------------------------------
 * Built-in scalar functions (each is already the fused composition, Sec. 2.1.2):
 *   "hmlstm_update" N=12 (f i o g c h z z_below b_f b_i b_o b_g) -> (c', h');
 *                   the cell update of Sec. 3.1 / 3.2.3: FLUSH if z == 1, COPY if
 *                   z == 0 and z_below == 0, UPDATE otherwise; h' = sigma(o) tanh(c')
 *                   except COPY (h' = h); biases add to their gate's pre-activation.
 *                   z, z_below are control inputs (not differentiable).
 *                   branch id: 0 UPDATE, 1 COPY, 2 FLUSH.
 *   "update_c"      N=6 (c f i g z1 z2) -> c'; the paper's fused update (Sec. 3.2.3).
 *   "tanh_xy_b"     N=3 -> tanh(x*y + b)
 *   "branchy5"      N=5 (A B r s t): exp(-A)*B + r if A + s > t else log1p(A*A)*r - s;
 *                   branch id 1 = predicate true.
 *   "cos_x"         N=1 (the Dual example of Sec. 2.2.1), "scale_xt" N=2 (x*t),
 *   "pair3"         N=3 -> (x1*x2 + sin x3, x1/x2 - x3*x3)  (R^3 -> R^2, Sec. 2.2.2)
 *   "elementary4"   N=1 -> (exp x, log1p x, sigma x, tanh x): the elementary functions the other
 *                   ops are built from (for measuring their accuracy over their whole domain)
 *   "linear12"      N=12, the HM-LSTM argument list with trivial arithmetic:
 *                   (sum of the ten differentiable arguments + z*z_below,
 *                    f*c + i*h + o*g + b_f*b_i + b_o*b_g); for profiling memory behaviour.
 *   "prod_tanh_K"   K = 1..18: prod_i tanh(g(x_i)), g(x) = x if x > 1/2 else -x
 *                   (the arity study of Sec. 3.4.1); branch id = #{x_i > 1/2}.
 * Predicates read values only, so control flow contributes no derivative. */
int bcast_op_lookup(const char *name, int32_t *op_id);
int bcast_op_count(void);
const char *bcast_op_name(int32_t op_id); /* NULL if out of range */
/* nondiff_mask bit j set = argument j is a control input: it has no partial plane and
 * no gradient.  N_d = n_args - popcount(nondiff_mask). */
int bcast_op_info(int32_t op_id, int32_t *n_args, int32_t *n_outputs, uint32_t *nondiff_mask,
                  int32_t *n_branches);

/* What the op table knows about the M * N_d planes of an op, for callers that want a leaner
 * partial store: alias[k] == k: plane k has content of its own; alias[k] == j < k: plane k is
 * identical to plane j on every branch (e.g. a bias and the gate it is added to); alias[k] == -1:
 * plane k is zero on every branch.  `alias` receives M * N_d entries. */
int bcast_op_plane_alias(int32_t op_id, int32_t *alias);

/* ---- forward: values + Jacobian planes in one kernel (Sec. 2.2.2, Sec. 2.2.3) -----
 * args[n_args]      inputs (read).  Unified shape = per-dim maximum; every argument dim
 *                   must equal it or be 1 (else BCAST_ERR_SHAPE_MISMATCH).
 * outs[n_out]       the M outputs (written), each exactly of the unified shape.
 * partials[M*N_d]   planes d Y_i / d X_jd (written), unified shape, index i*N_d + jd
 *                   where jd counts differentiable arguments in argument order
 *                   (row = output, column = argument, as in the D(b) expansion of
 *                   Sec. 2.2.2).  A plane whose data pointer is NULL is not stored.
 *                   Two slots may be given the very same view where bcast_op_plane_alias
 *                   declares the planes identical (it is then written once); any other
 *                   sharing of a view is refused with BCAST_ERR_BAD_STRIDE.
 *                   `partials` itself may be NULL: values only.
 * branch_id         optional device buffer of E bytes (E = elements of the unified
 *                   shape), row-major over the unified shape as given (before any
 *                   internal dim merging); receives the branch taken per element.
 * Written views must not have zero strides on dims of extent > 1. */
int bcast_dual_forward(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                       int32_t n_out, const bcast_tensor *outs, const bcast_tensor *partials,
                       uint8_t *branch_id, void *stream, const bcast_dual_options *opt);
int bcast_dual_forward_plan(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                            int32_t n_out, const bcast_tensor *outs, const bcast_tensor *partials,
                            const uint8_t *branch_id, bcast_plan_info *info, const bcast_dual_options *opt);

/* ---- backward: adjoint x partial, summed over expanded dims (Table 1) --------------
 * Independent of the op.
 * adjoints[n_out]   upstream adjoints of the M outputs (read), all of one shape S.
 * partials[M*n_grads] the planes forward produced (read), shape S, index i*n_grads + jd.
 *                   A NULL data pointer stands for a plane of zeros (its products with the
 *                   adjoint are adjoint x 0: nothing for a finite adjoint, NaN for an infinite one).
 * grads[n_grads]    gradient of each differentiable argument (written), in THAT
 *                   ARGUMENT's shape: every dim equals S's or is 1 (or is a missing
 *                   trailing dim); where it is 1 and S's extent is larger, the products
 *                   sum_i adj_i * P_i,jd are summed over that dim.  A NULL data pointer
 *                   skips that gradient.
 * workspace         device scratch for the deterministic second reduction pass; at least
 *                   bcast_dual_backward_workspace(...) bytes, 16-byte aligned; may be
 *                   NULL when that is 0.  Contents on entry are ignored.
 * Products are formed and summed in double (fp32 data) or in double-double (fp64 data)
 * and rounded once; there are no atomics, so results do not depend on scheduling. */
size_t bcast_dual_backward_workspace(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                                     const bcast_tensor *partials, int32_t n_grads,
                                     const bcast_tensor *grads, const bcast_dual_options *opt);
int bcast_dual_backward(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                        const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                        void *workspace, size_t workspace_bytes, void *stream, const bcast_dual_options *opt);
int bcast_dual_backward_plan(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                             const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                             bcast_plan_info *info, const bcast_dual_options *opt);

/* ---- backward for callers that cannot allocate --------------------------------------------------
 * For callers that have no way to provide a workspace: code that runs while a HIP graph is being
 * captured, tight serving loops, harnesses that forbid hipMalloc.  The same call as
 * bcast_dual_backward -- same arguments otherwise, same kernels, same results bit for bit -- with the
 * scratch memory of the second reduction pass taken from an array of BCAST_NOALLOC_SCRATCH_BYTES that
 * is part of the library's device image (one copy per GPU, held until the process ends) instead of a
 * caller's buffer.  The call allocates and frees nothing on the device (no hipMalloc / hipFree, no
 * allocating library routine).
 *  - A call whose partial sums need more than BCAST_NOALLOC_SCRATCH_BYTES (what
 *    bcast_dual_backward_workspace reports for the same arguments and options) returns
 *    BCAST_ERR_WORKSPACE_TOO_SMALL and launches nothing; every benchmark configuration needs under 6 MiB.
 *  - The device of `stream` must be the current device.  The first call on a device looks the array's
 *    address up (hipGetSymbolAddress) and keeps it; make that first call outside graph capture.
 *  - All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *    different threads) race on it and must be serialised by the caller.  Nothing has to be cleared
 *    between calls: every partial sum the second pass reads is written by the main pass of the same call. */
#define BCAST_NOALLOC_SCRATCH_BYTES (16u << 20)
int bcast_dual_backward_noalloc(bcast_dtype dt, int32_t n_out, const bcast_tensor *adjoints,
                                const bcast_tensor *partials, int32_t n_grads, const bcast_tensor *grads,
                                void *stream, const bcast_dual_options *opt);

/* ---- backward without cached planes: D applied in the reverse pass (Sec. 2.2.3, last paragraph) ----
 * The other side of the paper's memory/compute trade-off: nothing is kept between the passes
 * (the forward pass is then called with partials == NULL).  One kernel reads the op's arguments
 * and the adjoints, evaluates b on dual numbers again and reduces sum_i adj_i * dY_i/dX_jd into
 * each gradient exactly as bcast_dual_backward does.
 * args[n_args] as in forward; adjoints[n_out] of the unified shape; grads[n_grads = N_d] in their
 * argument's shape (NULL data: skipped; any other shape: BCAST_ERR_OUTPUT_SHAPE_MISMATCH).  Available for problems that merge to at most three dims
 * with unit inner stride (the tiled kernels), for every op (the prod_tanh_K family only where all
 * full-shape views share one row stride); otherwise BCAST_ERR_UNSUPPORTED.  Workspace rules as for bcast_dual_backward. */
size_t bcast_dual_backward_recompute_workspace(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                               int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                               const bcast_tensor *grads, const bcast_dual_options *opt);
int bcast_dual_backward_recompute(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                  int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                  const bcast_tensor *grads, void *workspace, size_t workspace_bytes, void *stream,
                                  const bcast_dual_options *opt);
/* How that call would be mapped (no launch); `specialized` = 1 when the kernel compiled for the op's
 * usual broadcast pattern runs (every argument's form fixed at compile time). */
int bcast_dual_backward_recompute_plan(int32_t op_id, bcast_dtype dt, int32_t n_args, const bcast_tensor *args,
                                       int32_t n_out, const bcast_tensor *adjoints, int32_t n_grads,
                                       const bcast_tensor *grads, bcast_plan_info *info, const bcast_dual_options *opt);

/* ---- unfused comparison: one kernel per primitive, reverse mode (Sec. 3.2.1, 3.2.2) -----------
 * Not the method: the comparison system the paper measures it against, written from the math.  The op's
 * scalar function becomes a chain of whole-array primitives (add, mul, sigmoid, tanh, exp, log1p, compare,
 * select, ...), each a kernel launch with its result in a temporary; every branch is computed for every
 * element and chosen by select; the reverse pass applies each primitive's own derivative rule, again one
 * kernel per rule, and sums a broadcast argument's gradient over its expanded dims with a reduction kernel.
 * For timing beside bcast_dual_forward + bcast_dual_backward; available for "hmlstm_update", "update_c",
 * "tanh_xy_b" and "branchy5" (else BCAST_ERR_UNSUPPORTED).
 * Every array is contiguous, row major, [rows x cols]; arg_kind[j] says what argument j is.  The gates,
 * cell and hidden state of the two cell updates, and A and B of branchy5, must be full arrays.
 * outs[n_out] (written), adjoints[n_out] (read): full arrays.  grads[n_grads = N_d] (written): each in its
 * argument's shape.  workspace: at least bcast_unfused_workspace(...) bytes, 256-byte aligned.
 * n_kernels (may be NULL) receives the number of kernels the call enqueued. */
enum { BCAST_UNFUSED_FULL = 0, BCAST_UNFUSED_ROW_VECTOR = 1 /* [1 x cols] */, BCAST_UNFUSED_COL_VECTOR = 2 /* [rows x 1] */,
       BCAST_UNFUSED_SCALAR = 3 };
size_t bcast_unfused_workspace(int32_t op_id, bcast_dtype dt, int64_t rows, int64_t cols);
int bcast_unfused_step(int32_t op_id, bcast_dtype dt, int64_t rows, int64_t cols, int32_t n_args, const void *const *args,
                       const int32_t *arg_kind, int32_t n_out, void *const *outs, const void *const *adjoints, int32_t n_grads,
                       void *const *grads, void *workspace, size_t workspace_bytes, void *stream, int32_t *n_kernels);

/* ---- misc ---------------------------------------------------------------------- */
const char *bcast_status_string(int status);

/* Partial-storage layout.  The planes of one call (outputs, the M x N_d partials, the
 * gradients, and ideally the arguments too) are streamed side by side, every wavefront
 * touching the same offset of each.  If the planes start a large power of two apart, those
 * accesses land on the same HBM channel; measured on MI355X, 29 written planes of 16 MiB move
 * at 4.0 TB/s when they start 16 MiB apart and at 5.7 TB/s when each plane is shifted by one
 * more 4 KiB page than its predecessor (7 read + 22 written planes: 4.7 against 5.2 TB/s).  This helper lays n_planes of plane_bytes each out
 * in one slab that way: offsets[k] (bytes, 256-byte aligned) is where plane k starts;
 * returns the slab size in bytes (offsets may be NULL to query only the size).  Using it is
 * optional: any non-overlapping views are accepted by forward and backward. */
size_t bcast_dual_slab_layout(size_t plane_bytes, int32_t n_planes, size_t *offsets);

/* Streaming probe for roofline calibration: fp32 planes are cut into chunks of 1024 floats
 * (4 KiB); one 256-lane block reads chunk b of each of the n_in input planes with 16-byte
 * loads, adds them, and writes chunk b of each of the n_out output planes -- the access
 * pattern of the tiled kernels with no arithmetic to speak of.  Chunk b of plane k starts at
 * plane[k] + b * chunk_stride[k] floats (1024 = a dense plane; larger = planes interleaved in
 * one buffer).  in/out and the stride arrays are HOST arrays (at most 32 entries each) of
 * DEVICE pointers (16-byte aligned) and strides (multiples of 4; output strides >= 1024).
 * n_in = 1, n_out = 1 is a plain copy, used to scale profiler byte counters.  The options
 * reverse_tiles (1 = chunks last to first, else first to last), probe_nt_loads and probe_lds_kib apply. */
int bcast_dual_stream_probe(int32_t n_in, const void *const *in, const int64_t *in_chunk_stride, int32_t n_out,
                            void *const *out, const int64_t *out_chunk_stride, int64_t n_chunks, void *stream,
                            const bcast_dual_options *opt);

#ifdef __cplusplus
}
#endif
#endif /* BCAST_DUAL_H */
