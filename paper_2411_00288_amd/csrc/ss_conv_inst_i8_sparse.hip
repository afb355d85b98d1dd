// Convolution kernels for i8 operands, 2:4-sparse weight operand.
#define SS_INST_NAME i8_sparse
#define SS_INST_DT SS_I8
#define SS_INST_SPARSE true
#define SS_INST_FUSED 0
#include "ss_conv_inst.h"
