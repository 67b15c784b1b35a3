// Device implementation of the counter-based synthetic tensor generator (gfx950).
//
// Same definition as generator.py / synth_host.c.  It only fills input tensors
// in HBM (the large workloads' weights do not fit in host memory); it holds no
// MoE arithmetic and is not part of the MoE library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__device__ __forceinline__ double variate(uint64_t key, uint64_t i) {
    int64_t s = 0;
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        uint64_t h = mix64(key + (3ULL * i + (uint64_t)m + 1ULL) * GOLDEN);
        s += (int64_t)(h & 0xFFFF) + (int64_t)((h >> 16) & 0xFFFF) + (int64_t)((h >> 32) & 0xFFFF) +
             (int64_t)(h >> 48);
    }
    return (double)(2 * s - 12 * 65535) / 131072.0;
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DTYPE>
__global__ void __launch_bounds__(256) synth_fill_kernel(void* __restrict__ out, uint64_t key, uint64_t start,
                                                         uint64_t count, double sigma) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t n = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; n < count; n += stride) {
        float v = (float)(sigma * variate(key, start + n));
        if (DTYPE == 0) ((float*)out)[n] = v;
        else ((uint16_t*)out)[n] = f32_to_bf16(v);
    }
}

static uint64_t host_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

// out: DEVICE pointer to `count` elements.  dtype 0 = fp32, 1 = bf16.  Asynchronous on `stream`.
// Returns 0 on success, -1 bad argument, -2 launch failure.
extern "C" int lexi_synth_fill_device(void* out, int dtype, uint64_t seed, uint64_t tid, uint64_t start,
                                      uint64_t count, double sigma, void* stream) {
    if ((dtype != 0 && dtype != 1) || (out == nullptr && count != 0)) return -1;
    if (count == 0) return 0;
    const uint64_t key = host_mix64(seed ^ host_mix64(tid + GOLDEN));
    uint64_t blocks = (count + 255) / 256;
    if (blocks > 256ULL * 64ULL) blocks = 256ULL * 64ULL;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == 0) hipLaunchKernelGGL(synth_fill_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, s, out, key, start, count, sigma);
    else hipLaunchKernelGGL(synth_fill_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, s, out, key, start, count, sigma);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}
