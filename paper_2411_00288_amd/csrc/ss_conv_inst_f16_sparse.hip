// Convolution kernels for f16 operands, 2:4-sparse weight operand.
#define SS_INST_NAME f16_sparse
#define SS_INST_DT SS_F16
#define SS_INST_SPARSE true
#define SS_INST_FUSED 1
#include "ss_conv_inst.h"
