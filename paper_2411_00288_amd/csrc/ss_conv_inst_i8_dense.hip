// Convolution kernels for i8 operands, dense weight operand (the twin).
#define SS_INST_NAME i8_dense
#define SS_INST_DT SS_I8
#define SS_INST_SPARSE false
#define SS_INST_FUSED 0
#include "ss_conv_inst.h"
