// forward kernels for bf16 storage, head_dim 16
#define SDFP_INST_WT bf16_t
#define SDFP_INST_HD 16
#include "sdfp_fwd_inst.hip.h"
