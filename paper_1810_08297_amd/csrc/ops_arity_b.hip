// Forward and recompute kernels of the arity-study family, arities 11..15.
#include "fwd_kernels.h"
#include "recompute_kernels.h"
BD_DEFINE_OP(bd::OpProdTanh<11>, prod_tanh_11)
BD_DEFINE_OP(bd::OpProdTanh<12>, prod_tanh_12)
BD_DEFINE_OP(bd::OpProdTanh<13>, prod_tanh_13)
BD_DEFINE_OP(bd::OpProdTanh<14>, prod_tanh_14)
BD_DEFINE_OP(bd::OpProdTanh<15>, prod_tanh_15)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<11>, prod_tanh_11)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<12>, prod_tanh_12)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<13>, prod_tanh_13)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<14>, prod_tanh_14)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<15>, prod_tanh_15)
