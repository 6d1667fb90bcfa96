// Device fill for the synthetic-tensor recipe defined in gen.py: lets a test or benchmark create
// multi-GB random-init weights directly in HBM.  Not part of the decode library; no method arithmetic.
#include <hip/hip_runtime.h>
#include <stdint.h>

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__device__ __forceinline__ float synth_value(uint64_t seed, uint64_t tid, uint64_t idx, float scale) {
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * ((tid << 40) + idx));
    int s = 0;
#pragma unroll
    for (int b = 0; b < 8; ++b) s += (int)((z >> (8 * b)) & 0xFF);
    return __fmul_rn((float)(s - 1020), scale);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

__global__ void fill_f32(float *out, uint64_t seed, uint64_t tid, uint64_t n, float scale) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        out[i] = synth_value(seed, tid, i, scale);
}

__global__ void fill_bf16(uint16_t *out, uint64_t seed, uint64_t tid, uint64_t n, float scale) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        out[i] = f32_to_bf16_rne(synth_value(seed, tid, i, scale));
}

__global__ void fill_const_f32(float *out, uint64_t n, float v) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x)
        out[i] = v;
}

extern "C" int synth_fill_device(void *dev_out, int dtype, uint64_t seed, uint64_t tid, uint64_t n, float scale,
                                 void *stream) {
    if (n == 0) return 0;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == 0)
        hipLaunchKernelGGL(fill_f32, dim3((unsigned)blocks), dim3(256), 0, st, (float *)dev_out, seed, tid, n, scale);
    else
        hipLaunchKernelGGL(fill_bf16, dim3((unsigned)blocks), dim3(256), 0, st, (uint16_t *)dev_out, seed, tid, n, scale);
    return (int)hipGetLastError();
}

extern "C" int synth_fill_const_device(float *dev_out, uint64_t n, float v, void *stream) {
    if (n == 0) return 0;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_const_f32, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, dev_out, n, v);
    return (int)hipGetLastError();
}
