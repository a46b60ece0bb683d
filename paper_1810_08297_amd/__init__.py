"""bcast_dual: mixed-mode differentiation of fused broadcasts on MI355X (gfx950).

The product is the C-ABI library (include/bcast_dual.h, csrc/); this package is its
thin Python binding plus buffer-allocation helpers and the seeded workload generators.
"""
from .binding import (  # noqa: F401
    BcastError, BcastTensor, PlanInfo, Options, F32, F64, LIB_PATH, EXPORTS,
    bcast_op_lookup, bcast_op_count, bcast_op_name, bcast_op_info, bcast_op_plane_alias, diff_arg_indices,
    bcast_dual_forward, bcast_dual_forward_plan, bcast_dual_backward_workspace,
    bcast_dual_backward, bcast_dual_backward_plan, bcast_dual_backward_noalloc, NOALLOC_SCRATCH_BYTES, bcast_dual_stream_probe, bcast_dual_slab_layout, status_string, as_view, raw_view, PreparedForward, PreparedBackward, PreparedRecompute,
    bcast_dual_backward_recompute, bcast_dual_backward_recompute_workspace, bcast_dual_backward_recompute_plan,
    bcast_unfused_workspace, bcast_unfused_step,
)
from .helpers import ForwardBuffers, BackwardBuffers, alloc_forward, alloc_backward, alloc_planes, to_slab, alloc_recompute, LaunchTimer  # noqa: F401
from .autograd import broadcast  # noqa: F401
