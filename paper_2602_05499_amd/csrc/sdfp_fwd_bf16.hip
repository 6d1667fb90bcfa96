// the forward kernel for weights and KV cache stored as bf16_t (one translation unit per storage type so that
// the two compile in parallel)
#include "sdfp_forward.hip.h"
namespace sdfp {
template __global__ void k_forward<bf16_t, 0>(FwdArgs);
template __global__ void k_forward<bf16_t, 1>(FwdArgs);
template __global__ void k_forward<bf16_t, 2>(FwdArgs);
template __global__ void k_forward<bf16_t, 3>(FwdArgs);
}  // namespace sdfp
