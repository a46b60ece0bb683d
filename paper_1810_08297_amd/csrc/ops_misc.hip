// Forward kernels of the generic broadcast ops.
#include "fwd_kernels.h"
#include "recompute_kernels.h"
BD_DEFINE_OP(bd::OpTanhXyB, tanh_xy_b)
BD_DEFINE_OP(bd::OpBranchy5, branchy5)
BD_DEFINE_OP(bd::OpCosX, cos_x)
BD_DEFINE_OP(bd::OpScaleXt, scale_xt)
BD_DEFINE_OP(bd::OpPair3, pair3)
BD_DEFINE_OP(bd::OpLinear12, linear12)
BD_DEFINE_OP(bd::OpElementary4, elementary4)
BD_DEFINE_OP_RECOMPUTE(bd::OpTanhXyB, tanh_xy_b)
BD_DEFINE_OP_RECOMPUTE(bd::OpBranchy5, branchy5)
BD_DEFINE_OP_RECOMPUTE(bd::OpCosX, cos_x)
BD_DEFINE_OP_RECOMPUTE(bd::OpScaleXt, scale_xt)
BD_DEFINE_OP_RECOMPUTE(bd::OpPair3, pair3)
BD_DEFINE_OP_RECOMPUTE(bd::OpLinear12, linear12)
BD_DEFINE_OP_RECOMPUTE(bd::OpElementary4, elementary4)
