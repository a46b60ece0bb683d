// Forward kernels of the HM-LSTM cell-update ops.
#include "fwd_kernels.h"
#include "recompute_kernels.h"
BD_DEFINE_OP(bd::OpHmLstmUpdate, hmlstm_update)
BD_DEFINE_OP(bd::OpUpdateC, update_c)
BD_DEFINE_OP_RECOMPUTE(bd::OpHmLstmUpdate, hmlstm_update)
BD_DEFINE_OP_RECOMPUTE(bd::OpUpdateC, update_c)
