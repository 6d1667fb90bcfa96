// Explicit instantiations of the templated kernels, split over translation units so that they compile in
// parallel.  Included with SDFP_EXTERN = "extern" by the host code (declarations only) and with SDFP_EXTERN
// empty and SDFP_INST_WT / SDFP_INST_GROUP set by the per-group instantiation files.
#include "sdfp_forward.hip.h"   // common, GEMV, attention, one-launch forward (templates only)

namespace sdfp {
#define SDFP_INST_ONE(WT, MT, D)                                                                                   \
    SDFP_EXTERN template __global__ void k_forward<WT, MT, D>(FwdArgs);                                            \
    SDFP_EXTERN template __global__ void k_qkv<WT, MT, D>(QkvOp<WT, MT>, Rows, const DevState*, const float*,      \
                                                          const float*, float);                                    \
    SDFP_EXTERN template __global__ void k_resid<WT, MT, D>(ResidOp<WT, MT>, const float*);                        \
    SDFP_EXTERN template __global__ void k_gateup<WT, MT, D>(GateUpOp<WT, MT>, const float*, const float*, float); \
    SDFP_EXTERN template __global__ void k_head<WT, MT, D>(const WT*, const float*, const float*, float, int, int, \
                                                           int, HeadOut, DevState*);
#define SDFP_INST_G0(WT) SDFP_INST_ONE(WT, 1, 16) SDFP_INST_ONE(WT, 2, 16) SDFP_INST_ONE(WT, 3, 8)
#define SDFP_INST_G1(WT) SDFP_INST_ONE(WT, 4, 8) SDFP_INST_ONE(WT, 5, 8) SDFP_INST_ONE(WT, 6, 8)
#define SDFP_INST_G2(WT) SDFP_INST_ONE(WT, 7, 4) SDFP_INST_ONE(WT, 8, 4) SDFP_INST_ONE(WT, 9, 4)

#if defined(SDFP_INST_GROUP)
#if SDFP_INST_GROUP == 0
SDFP_INST_G0(SDFP_INST_WT)
#elif SDFP_INST_GROUP == 1
SDFP_INST_G1(SDFP_INST_WT)
#else
SDFP_INST_G2(SDFP_INST_WT)
#endif
#else
SDFP_INST_G0(float) SDFP_INST_G1(float) SDFP_INST_G2(float)
SDFP_INST_G0(bf16_t) SDFP_INST_G1(bf16_t) SDFP_INST_G2(bf16_t)
#endif
}  // namespace sdfp
