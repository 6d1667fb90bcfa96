// Explicit instantiation of the forward kernel for one storage type and one head_dim (all four roles): included by
// the sdfp_fwd_<type>_hd<n>.hip translation units, which only set SDFP_INST_WT and SDFP_INST_HD, so that the
// instances compile in parallel.
#include "sdfp_forward.hip.h"
namespace sdfp {
template __global__ void k_forward<SDFP_INST_WT, 0, attn_lpp(SDFP_INST_HD)>(FwdArgs);
template __global__ void k_forward<SDFP_INST_WT, 1, attn_lpp(SDFP_INST_HD)>(FwdArgs);
template __global__ void k_forward<SDFP_INST_WT, 2, attn_lpp(SDFP_INST_HD)>(FwdArgs);
template __global__ void k_forward<SDFP_INST_WT, 3, attn_lpp(SDFP_INST_HD)>(FwdArgs);
}  // namespace sdfp
