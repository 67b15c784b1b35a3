// Stage-1 top-k perturbation profiling (paper Algorithm 1), one iteration on one input X:
//     Delta_k = || f_moe(X; k) - f_moe(X; k_base) ||_F          for every k of a list, k <= k_base.
// The selection is a total order, so TopK_k is the first k slots of TopK_{k_base}; the gates of k are the baseline
// gates of those slots renormalised over them.  One routing pass and one pass of the expert GEMMs at k_base therefore
// serve every k:
//     Y_k[t] - Y_base[t] = sum_{s < k_base} ( [s < k] * g[t][s] / P_k[t] - g[t][s] ) * y_slot[t][s],
//     P_k[t] = g[t][0] + ... + g[t][k-1]   (ascending),
// and a shared expert, which adds the same vector to both outputs, drops out.  fp32 throughout, fixed summation
// orders (same bits on every run); the final sum over tokens and the square root are taken in fp64.
#include "kernels.hpp"

namespace lexi {

// One workgroup per token: squared norm of the difference vector for every listed k -> part[i][t].
__global__ void __launch_bounds__(256)
profile_diff_kernel(const float* __restrict__ y_slot, const int32_t* __restrict__ inv_perm, const float* __restrict__ gates,
                    int T, int d, int k_base, ProfileKList kl, float* __restrict__ part) {
    __shared__ float wave_part[4];
    const int t = blockIdx.x;
    const int32_t* ip = inv_perm + (size_t)t * k_base;
    const float* gt = gates + (size_t)t * k_base;
    for (int i = 0; i < kl.n; ++i) {
        const int k = kl.k[i];
        float sq = 0.0f;
        if (k != k_base) {                      // k == k_base: every coefficient is zero, Delta is exactly 0
            float pk = 0.0f;
            for (int s = 0; s < k; ++s) pk += gt[s];
            const float inv = 1.0f / pk;
            for (int j = threadIdx.x * 4; j < d; j += 256 * 4) {
                f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                for (int s = 0; s < k_base; ++s) {   // slot order
                    const float g = gt[s];
                    const float c = (s < k ? g * inv : 0.0f) - g;
                    const f32x4_t v = *(const f32x4_t*)(y_slot + (size_t)ip[s] * d + j);
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] = __builtin_fmaf(c, v[q], acc[q]);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) sq = __builtin_fmaf(acc[q], acc[q], sq);
            }
        }
        const float ws = wave_sum(sq);
        __syncthreads();                        // the previous k's wave_part has been read
        if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ws;
        __syncthreads();
        if (threadIdx.x == 0) part[(size_t)i * T + t] = ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];
    }
}

// One workgroup per listed k: sum of the T per-token squared norms in a fixed order (strided partial sums per thread,
// then the DPP tree and the four wave results in wave order), in fp64; delta = sqrt(sum).
__global__ void __launch_bounds__(256)
profile_reduce_kernel(const float* __restrict__ part, int T, float* __restrict__ delta) {
    __shared__ double wave_part[4];
    const float* p = part + (size_t)blockIdx.x * T;
    double s = 0.0;
    for (int t = threadIdx.x; t < T; t += 256) s += (double)p[t];
    // fixed-order tree over the 64 lanes (xor butterfly: every lane ends with the same sum)
    for (int off = 32; off >= 1; off >>= 1) {
        const int lo = __shfl_xor((int)(__double_as_longlong(s) & 0xFFFFFFFFll), off);
        const int hi = __shfl_xor((int)(__double_as_longlong(s) >> 32), off);
        s += __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
    }
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) delta[blockIdx.x] = (float)sqrt(((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3]);
}

hipError_t launch_profile(const ProfileArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(profile_diff_kernel, dim3(a.T), dim3(256), 0, s, a.y_slot, a.inv_perm, a.gates, a.T, a.d,
                       a.k_base, a.klist, a.part);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(profile_reduce_kernel, dim3(a.klist.n), dim3(256), 0, s, a.part, a.T, a.delta);
    return hipGetLastError();
}

}  // namespace lexi
