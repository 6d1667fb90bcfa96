// forward kernels for f32 storage, head_dim 16
#define SDFP_INST_WT float
#define SDFP_INST_HD 16
#include "sdfp_fwd_inst.hip.h"
