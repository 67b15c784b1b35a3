// Gate-weighted unpermute / combine (paper Sec. 2: y = sum_i G(x)_i * E_i(x)), the shared-expert term, and the
// sigmoid gate in front of a gated shared expert (evaluated inside the combine).  fp32, fixed slot order, no atomics: same bits on every run.
#include "kernels.hpp"

namespace lexi {

// One workgroup per token; each thread owns 4 consecutive output features per pass.  For a sigmoid-gated shared
// expert the workgroup first evaluates its token's gate coefficient 1 / (1 + exp(-(x[t] . w_sg))) itself (wave sums by
// DPP, the four wave results added in wave order), which saves a launch.
template <bool Y_BF16, bool X_BF16>
__global__ void __launch_bounds__(256)
combine_kernel(const float* __restrict__ y_slot, const int32_t* __restrict__ inv_perm, const float* __restrict__ gates,
               const float* __restrict__ y_shared, const void* __restrict__ x, const void* __restrict__ w_shared_gate,
               int d, int k, void* __restrict__ y) {
    __shared__ float wave_part[4];
    const int t = blockIdx.x;
    const int32_t* ip = inv_perm + (size_t)t * k;
    const float* gt = gates + (size_t)t * k;
    float coef = (y_shared != nullptr) ? 1.0f : 0.0f;
    if (y_shared != nullptr && w_shared_gate != nullptr) {
        float acc = 0.0f;
        for (int j = threadIdx.x; j < d; j += 256)
            acc = __builtin_fmaf(load_as_f32<X_BF16>(x, (size_t)t * d + j), load_as_f32<X_BF16>(w_shared_gate, (size_t)j), acc);
        const float ws = wave_sum(acc);
        if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ws;
        __syncthreads();
        const float z = ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];
        coef = 1.0f / (1.0f + __expf(-z));
    }
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

template <bool Y_BF16, bool X_BF16>
static void launch_combine_t(const CombineArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((combine_kernel<Y_BF16, X_BF16>), dim3(a.T), dim3(256), 0, s, a.y_slot, a.inv_perm, a.gates,
                       a.y_shared, a.x, a.w_shared_gate, a.d, a.k, a.y);
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s) {
    if (a.y_bf16) { if (a.x_bf16) launch_combine_t<true, true>(a, s); else launch_combine_t<true, false>(a, s); }
    else          { if (a.x_bf16) launch_combine_t<false, true>(a, s); else launch_combine_t<false, false>(a, s); }
    return hipGetLastError();
}

}  // namespace lexi
