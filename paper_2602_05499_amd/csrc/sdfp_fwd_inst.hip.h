// Explicit instantiation of the forward kernel for one storage type and one head_dim: prompt chunks, draft row,
// plain decode row, and one verify kernel per row count 2..9.  Included by the sdfp_fwd_<type>_hd<n>.hip
// translation units, which only set SDFP_INST_WT and SDFP_INST_HD, so that the instances compile in parallel.
#include "sdfp_forward.hip.h"
namespace sdfp {
#define SDFP_INST(ROLE, M) template __global__ void k_forward<SDFP_INST_WT, ROLE, attn_lpp(SDFP_INST_HD), M>(FwdArgs);
SDFP_INST(0, 0)
SDFP_INST(1, 1)
SDFP_INST(3, 1)
SDFP_INST(2, 2) SDFP_INST(2, 3) SDFP_INST(2, 4) SDFP_INST(2, 5) SDFP_INST(2, 6) SDFP_INST(2, 7) SDFP_INST(2, 8) SDFP_INST(2, 9)
#undef SDFP_INST
}  // namespace sdfp
