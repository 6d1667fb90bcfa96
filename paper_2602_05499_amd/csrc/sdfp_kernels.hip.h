// Device code of libsdfp for gfx950 (CDNA4, wave64), split by step of the hot path:
//   sdfp_common.hip.h   storage types, device-resident decode state, DPP reductions
//   sdfp_stream.hip.h   weight-streaming projections on the matrix cores with fused norm / RoPE+KV / SiLU /
//                       residual / arg-max, and the loader that prefetches weights across phase boundaries
//   sdfp_attn.hip.h     causal attention of M <= 16 rows over the contiguous cache
//   sdfp_forward.hip.h  the whole forward as one persistent kernel with grid barriers
//   sdfp_select.hip.h   token selection: draft draws, accept/reject, resample, rollback
#pragma once
#include "sdfp_common.hip.h"
#include "sdfp_stream.hip.h"
#include "sdfp_attn.hip.h"
#include "sdfp_forward.hip.h"
#include "sdfp_select.hip.h"
