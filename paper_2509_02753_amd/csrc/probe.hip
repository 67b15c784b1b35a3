// Measured ceilings of the device, for the roofline report: what the matrix cores and the HBM sustain in plain loops
// with nothing else going on.  The caller times the launches with events; nothing here is on the MoE path.
#include "../../include/lexi_probe.h"
#include "common.hpp"

namespace lexi {

// Every wave keeps 2 x 8 accumulator blocks of v_mfma_f32_32x32x16_bf16 busy on fragments read once from `operands`
// (so the operand bits, and with them the switching activity and the clock the chip sustains, are the caller's).
__global__ void __launch_bounds__(256, 1)
probe_mfma_kernel(const bf16x8_t* __restrict__ operands, float* __restrict__ sink, int iters) {
    constexpr int FB = 2, TB = 8;
    f32x16_t acc[FB][TB];
#pragma unroll
    for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    bf16x8_t a[FB], b[TB];
#pragma unroll
    for (int i = 0; i < FB; ++i) a[i] = operands[threadIdx.x + 256 * i];
#pragma unroll
    for (int j = 0; j < TB; ++j) b[j] = operands[threadIdx.x + 256 * (FB + j)];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < FB; ++i)
#pragma unroll
            for (int j = 0; j < TB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        asm volatile("" ::: "memory");
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j) s += acc[i][j][0] + acc[i][j][15];
    if (s == 12345.678f) sink[threadIdx.x] = s;   // keeps the loop alive; practically never true
}

// Streaming read: a grid-stride sweep of 16-byte loads, eight in flight per lane.
__global__ void __launch_bounds__(256)
probe_read_kernel(const u32x4_t* __restrict__ src, size_t n_vec, uint32_t* __restrict__ sink) {
    u32x4_t s = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n_vec; i += 8 * stride) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s ^= v[u];
    }
    for (; i < n_vec; i += stride) s ^= src[i];
    if ((s[0] ^ s[1] ^ s[2] ^ s[3]) == 0x9E3779B9u) sink[threadIdx.x] = s[0];
}

}  // namespace lexi

extern "C" {

lexi_status lexi_probe_mfma_bf16(const void* operands, void* sink, int32_t iters, int32_t workgroups, void* hip_stream) {
    if (!operands || !sink) return LEXI_ERR_NULL;
    if (iters < 1 || workgroups < 1 || (((uintptr_t)operands | (uintptr_t)sink) & 15u)) return LEXI_ERR_SHAPE;
    hipLaunchKernelGGL(lexi::probe_mfma_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream,
                       (const lexi::bf16x8_t*)operands, (float*)sink, iters);
    return hipGetLastError() == hipSuccess ? LEXI_OK : LEXI_ERR_LAUNCH;
}

lexi_status lexi_probe_hbm_read(const void* src, size_t bytes, void* sink, void* hip_stream) {
    if (!src || !sink) return LEXI_ERR_NULL;
    if (bytes < 16 || (((uintptr_t)src | (uintptr_t)sink) & 15u)) return LEXI_ERR_SHAPE;
    hipLaunchKernelGGL(lexi::probe_read_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)hip_stream,
                       (const lexi::u32x4_t*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? LEXI_OK : LEXI_ERR_LAUNCH;
}

}  // extern "C"
