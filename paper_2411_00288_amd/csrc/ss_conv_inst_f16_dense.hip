// Convolution kernels for f16 operands, dense weight operand (the twin).
#define SS_INST_NAME f16_dense
#define SS_INST_DT SS_F16
#define SS_INST_SPARSE false
#define SS_INST_FUSED 1
#include "ss_conv_inst.h"
