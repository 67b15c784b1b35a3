// Gate-weighted unpermute / combine (paper Sec. 2: y = sum_i G(x)_i * E_i(x)), the shared-expert term, and the
// sigmoid gate in front of a gated shared expert.  fp32, fixed slot order, no atomics: same bits on every run.
#include "kernels.hpp"

namespace lexi {

// One workgroup per token; each thread owns 4 consecutive output features per pass.
template <bool Y_BF16>
__global__ void __launch_bounds__(256)
combine_kernel(const float* __restrict__ y_slot, const int32_t* __restrict__ inv_perm, const float* __restrict__ gates,
               const float* __restrict__ y_shared, const float* __restrict__ shared_coef, int d, int k,
               void* __restrict__ y) {
    const int t = blockIdx.x;
    const int32_t* ip = inv_perm + (size_t)t * k;
    const float* gt = gates + (size_t)t * k;
    const float coef = (y_shared != nullptr) ? (shared_coef ? shared_coef[t] : 1.0f) : 0.0f;
    for (int j = threadIdx.x * 4; j < d; j += 256 * 4) {
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s = 0; s < k; ++s) {  // slot order = rank order
            const f32x4_t v = *(const f32x4_t*)(y_slot + (size_t)ip[s] * d + j);
            const float g = gt[s];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(g, v[i], acc[i]);
        }
        if (y_shared != nullptr) {
            const f32x4_t v = *(const f32x4_t*)(y_shared + (size_t)t * d + j);
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(coef, v[i], acc[i]);
        }
        if (Y_BF16) {
            u32x2_t pk;
            pk[0] = pack_bf16x2(acc[0], acc[1]);
            pk[1] = pack_bf16x2(acc[2], acc[3]);
            *(u32x2_t*)((bf16_t*)y + (size_t)t * d + j) = pk;
        } else {
            *(f32x4_t*)((float*)y + (size_t)t * d + j) = acc;
        }
    }
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s) {
    if (a.y_bf16)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(a.T), dim3(256), 0, s, a.y_slot, a.inv_perm, a.gates, a.y_shared,
                           a.shared_coef, a.d, a.k, a.y);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(a.T), dim3(256), 0, s, a.y_slot, a.inv_perm, a.gates, a.y_shared,
                           a.shared_coef, a.d, a.k, a.y);
    return hipGetLastError();
}

// coef[t] = 1 / (1 + exp(-(x[t] . w))): one wave per token, lanes stride the hidden dimension.
template <bool IS_BF16>
__global__ void __launch_bounds__(256)
shared_gate_kernel(const void* __restrict__ x, const void* __restrict__ w, int T, int d, float* __restrict__ coef) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int lane = threadIdx.x & 63;
    float acc = 0.0f;
    for (int j = lane; j < d; j += 64)
        acc = __builtin_fmaf(load_as_f32<IS_BF16>(x, (size_t)t * d + j), load_as_f32<IS_BF16>(w, (size_t)j), acc);
    const float z = wave_sum(acc);
    if (lane == 0) coef[t] = 1.0f / (1.0f + __expf(-z));
}

hipError_t launch_shared_gate(const void* x, const void* w, bool is_bf16, int T, int d, float* coef, hipStream_t s) {
    const dim3 grid((T + 3) / 4);
    if (is_bf16)
        hipLaunchKernelGGL(shared_gate_kernel<true>, grid, dim3(256), 0, s, x, w, T, d, coef);
    else
        hipLaunchKernelGGL(shared_gate_kernel<false>, grid, dim3(256), 0, s, x, w, T, d, coef);
    return hipGetLastError();
}

}  // namespace lexi
