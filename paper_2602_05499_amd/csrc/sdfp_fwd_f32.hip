// the forward kernel for weights and KV cache stored as float (one translation unit per storage type so that
// the two compile in parallel)
#include "sdfp_forward.hip.h"
namespace sdfp {
template __global__ void k_forward<float, 0>(FwdArgs);
template __global__ void k_forward<float, 1>(FwdArgs);
template __global__ void k_forward<float, 2>(FwdArgs);
template __global__ void k_forward<float, 3>(FwdArgs);
}  // namespace sdfp
