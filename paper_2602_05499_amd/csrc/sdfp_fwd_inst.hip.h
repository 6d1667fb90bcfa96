// Explicit instantiation of the forward kernel for one storage type and one head_dim: prompt chunks, draft row,
// plain decode row, and one verify kernel per row count 2..9 -- the decode kernels twice, with and without turns
// that go on into the next tile.  Included by the sdfp_fwd_<type>_hd<n>.hip translation units, which only set
// SDFP_INST_WT and SDFP_INST_HD, so that the instances compile in parallel.
#include "sdfp_forward.hip.h"
namespace sdfp {
#define SDFP_INST(ROLE, M, SPAN) \
    template __global__ void k_forward<SDFP_INST_WT, ROLE, attn_lpp(SDFP_INST_HD), M, SPAN>(FwdArgs);
#define SDFP_INST_DECODE(SPAN)                                                                          \
    SDFP_INST(1, 1, SPAN) SDFP_INST(3, 1, SPAN)                                                          \
    SDFP_INST(2, 2, SPAN) SDFP_INST(2, 3, SPAN) SDFP_INST(2, 4, SPAN) SDFP_INST(2, 5, SPAN)              \
    SDFP_INST(2, 6, SPAN) SDFP_INST(2, 7, SPAN) SDFP_INST(2, 8, SPAN) SDFP_INST(2, 9, SPAN)
SDFP_INST(0, 0, false)
SDFP_INST_DECODE(false)
SDFP_INST_DECODE(true)
#undef SDFP_INST_DECODE
#undef SDFP_INST
}  // namespace sdfp
