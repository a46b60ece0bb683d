// Forward kernels of the arity-study family, arities 1..10.
#include "fwd_kernels.h"
BD_DEFINE_OP(bd::OpProdTanh<1>, prod_tanh_1)
BD_DEFINE_OP(bd::OpProdTanh<2>, prod_tanh_2)
BD_DEFINE_OP(bd::OpProdTanh<3>, prod_tanh_3)
BD_DEFINE_OP(bd::OpProdTanh<4>, prod_tanh_4)
BD_DEFINE_OP(bd::OpProdTanh<5>, prod_tanh_5)
BD_DEFINE_OP(bd::OpProdTanh<6>, prod_tanh_6)
BD_DEFINE_OP(bd::OpProdTanh<7>, prod_tanh_7)
BD_DEFINE_OP(bd::OpProdTanh<8>, prod_tanh_8)
BD_DEFINE_OP(bd::OpProdTanh<9>, prod_tanh_9)
BD_DEFINE_OP(bd::OpProdTanh<10>, prod_tanh_10)
