// Convolution kernels for f8 operands, 2:4-sparse weight operand.
#define SS_INST_NAME f8_sparse
#define SS_INST_DT SS_F8
#define SS_INST_SPARSE true
#define SS_INST_FUSED 0
#include "ss_conv_inst.h"
