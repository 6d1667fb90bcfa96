// forward kernels for bf16 storage, head_dim 64
#define SDFP_INST_WT bf16_t
#define SDFP_INST_HD 64
#include "sdfp_fwd_inst.hip.h"
