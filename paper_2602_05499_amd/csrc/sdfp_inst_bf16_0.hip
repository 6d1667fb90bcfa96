// kernel instantiations: storage type bf16, row-count group 0 (see sdfp_inst.hip.h)
#define SDFP_EXTERN
#define SDFP_INST_WT bf16_t
#define SDFP_INST_GROUP 0
#include "sdfp_inst.hip.h"
