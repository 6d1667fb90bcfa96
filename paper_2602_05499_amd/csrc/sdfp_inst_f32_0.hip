// kernel instantiations: storage type f32, row-count group 0 (see sdfp_inst.hip.h)
#define SDFP_EXTERN
#define SDFP_INST_WT float
#define SDFP_INST_GROUP 0
#include "sdfp_inst.hip.h"
