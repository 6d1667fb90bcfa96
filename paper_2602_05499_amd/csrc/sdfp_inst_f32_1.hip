// kernel instantiations: storage type f32, row-count group 1 (see sdfp_inst.hip.h)
#define SDFP_EXTERN
#define SDFP_INST_WT float
#define SDFP_INST_GROUP 1
#include "sdfp_inst.hip.h"
