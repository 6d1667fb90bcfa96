// forward kernels for f32 storage, head_dim 64
#define SDFP_INST_WT float
#define SDFP_INST_HD 64
#include "sdfp_fwd_inst.hip.h"
