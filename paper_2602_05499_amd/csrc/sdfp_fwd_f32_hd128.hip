// forward kernels for f32 storage, head_dim 128
#define SDFP_INST_WT float
#define SDFP_INST_HD 128
#include "sdfp_fwd_inst.hip.h"
