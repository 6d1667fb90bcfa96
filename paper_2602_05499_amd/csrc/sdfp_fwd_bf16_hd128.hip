// forward kernels for bf16 storage, head_dim 128
#define SDFP_INST_WT bf16_t
#define SDFP_INST_HD 128
#include "sdfp_fwd_inst.hip.h"
