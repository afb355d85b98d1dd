// Convolution kernels for f8 operands, dense weight operand (the twin).
#define SS_INST_NAME f8_dense
#define SS_INST_DT SS_F8
#define SS_INST_SPARSE false
#define SS_INST_FUSED 0
#include "ss_conv_inst.h"
