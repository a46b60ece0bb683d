// Forward and recompute kernels of the arity-study family, arities 16..18.
#include "fwd_kernels.h"
#include "recompute_kernels.h"
BD_DEFINE_OP(bd::OpProdTanh<16>, prod_tanh_16)
BD_DEFINE_OP(bd::OpProdTanh<17>, prod_tanh_17)
BD_DEFINE_OP(bd::OpProdTanh<18>, prod_tanh_18)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<16>, prod_tanh_16)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<17>, prod_tanh_17)
BD_DEFINE_OP_RECOMPUTE(bd::OpProdTanh<18>, prod_tanh_18)
