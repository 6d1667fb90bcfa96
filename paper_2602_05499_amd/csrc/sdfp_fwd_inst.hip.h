// Explicit instantiation of the forward kernel for one storage type and one head_dim: prompt chunks, draft row,
// plain decode row, and one verify kernel per row count 2..9 -- the decode kernels four times: with and without turns
// that go on into the next tile, for contexts of at most 8 attention splits and for longer ones.  Included by the sdfp_fwd_<type>_hd<n>.hip translation units, which only set
// SDFP_INST_WT and SDFP_INST_HD, so that the instances compile in parallel.
#include "sdfp_forward.hip.h"
namespace sdfp {
#define SDFP_INST(ROLE, M, SPAN, LONGCTX) \
    template __global__ void k_forward<SDFP_INST_WT, ROLE, attn_lpp(SDFP_INST_HD), M, SPAN, LONGCTX>(FwdArgs);
#define SDFP_INST_DECODE(SPAN, LONGCTX)                                                                                   \
    SDFP_INST(1, 1, SPAN, LONGCTX) SDFP_INST(3, 1, SPAN, LONGCTX)                                                          \
    SDFP_INST(2, 2, SPAN, LONGCTX) SDFP_INST(2, 3, SPAN, LONGCTX) SDFP_INST(2, 4, SPAN, LONGCTX) SDFP_INST(2, 5, SPAN, LONGCTX) \
    SDFP_INST(2, 6, SPAN, LONGCTX) SDFP_INST(2, 7, SPAN, LONGCTX) SDFP_INST(2, 8, SPAN, LONGCTX) SDFP_INST(2, 9, SPAN, LONGCTX)
SDFP_INST(0, 0, false, true)
SDFP_INST_DECODE(false, false)
SDFP_INST_DECODE(true, false)
SDFP_INST_DECODE(false, true)
SDFP_INST_DECODE(true, true)
#undef SDFP_INST_DECODE
#undef SDFP_INST
}  // namespace sdfp
