// Gate-weighted unpermute / combine (paper Sec. 2: y = sum_i G(x)_i * E_i(x)), the shared-expert term, and the
// sigmoid gate in front of a gated shared expert (evaluated inside the combine).  fp32, fixed slot order, no atomics: same bits on every run.
#include "kernels.hpp"

namespace lexi {

// u = h * inv rounded to the layer dtype, four consecutive elements (the chained stack's normalised MoE input).
template <bool U_BF16>
__device__ __forceinline__ void store_normalised(void* u, size_t idx, const f32x4_t& v, float inv) {
    if (U_BF16) {
        u32x2_t pk;
        pk[0] = pack_bf16x2(v[0] * inv, v[1] * inv);
        pk[1] = pack_bf16x2(v[2] * inv, v[3] * inv);
        *(u32x2_t*)((bf16_t*)u + idx) = pk;
    } else {
        f32x4_t o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = v[i] * inv;
        *(f32x4_t*)((float*)u + idx) = o;
    }
}

// One workgroup per token; each thread owns 4 consecutive output features per pass.  For a sigmoid-gated shared
// expert the workgroup first evaluates its token's gate coefficient 1 / (1 + exp(-(x[t] . w_sg))) itself (wave sums by
// DPP, the four wave results added in wave order), which saves a launch.
// Chained stack: `residual` (the hidden state) is added to the block's output, and with `u_next` the same workgroup
// also writes the NEXT block's normalised input from the row it has just produced -- the sum of squares in exactly
// the order rmsnorm_kernel uses, so either route gives the same bits.  (x and u_next may be the same buffer: a
// workgroup reads its row of x before it writes its row of u_next.)
template <bool Y_BF16, bool X_BF16>
__global__ void __launch_bounds__(256)
combine_kernel(const float* __restrict__ y_slot, const int32_t* __restrict__ inv_perm, const float* __restrict__ gates,
               const float* __restrict__ y_shared, const void* x, const void* __restrict__ w_shared_gate,
               const float* residual, int d, int k, void* y, void* u_next, float eps, int slot_planes,
               size_t slot_plane_stride, int shared_planes, size_t shared_plane_stride) {
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
    float ss = 0.0f;
    for (int j = threadIdx.x * 4; j < d; j += 256 * 4) {
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int s = 0; s < k; ++s) {  // slot order = rank order
            f32x4_t v = *(const f32x4_t*)(y_slot + (size_t)ip[s] * d + j);
            if (slot_planes > 1) {   // the down GEMM's reduction was cut in two: the halves are added first
                const f32x4_t v1 = *(const f32x4_t*)(y_slot + slot_plane_stride + (size_t)ip[s] * d + j);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = v[i] + v1[i];
            }
            const float g = gt[s];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(g, v[i], acc[i]);
        }
        if (y_shared != nullptr) {
            f32x4_t v = *(const f32x4_t*)(y_shared + (size_t)t * d + j);
            if (shared_planes > 1) {
                const f32x4_t v1 = *(const f32x4_t*)(y_shared + shared_plane_stride + (size_t)t * d + j);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = v[i] + v1[i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_fmaf(coef, v[i], acc[i]);
        }
        if (residual != nullptr) {   // chained stack: the hidden state plus this block's output (may alias y: same element)
            const f32x4_t h = *(const f32x4_t*)(residual + (size_t)t * d + j);
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = h[i] + acc[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(acc[i], acc[i], ss);
        if (Y_BF16) {
            u32x2_t pk;
            pk[0] = pack_bf16x2(acc[0], acc[1]);
            pk[1] = pack_bf16x2(acc[2], acc[3]);
            *(u32x2_t*)((bf16_t*)y + (size_t)t * d + j) = pk;
        } else {
            *(f32x4_t*)((float*)y + (size_t)t * d + j) = acc;
        }
    }
    if (Y_BF16 || u_next == nullptr) return;   // (the chained stack keeps its hidden state in fp32)
    __syncthreads();                            // wave_part may still be read for the gate coefficient
    const float ws = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ws;
    __syncthreads();
    const float total = ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];
    const float inv = 1.0f / sqrtf(total / (float)d + eps);
    for (int j = threadIdx.x * 4; j < d; j += 256 * 4) {
        const f32x4_t v = *(const f32x4_t*)((const float*)y + (size_t)t * d + j);   // this thread's own stores
        store_normalised<X_BF16>(u_next, (size_t)t * d + j, v, inv);
    }
}

template <bool Y_BF16, bool X_BF16>
static void launch_combine_t(const CombineArgs& a, hipStream_t s) {
    hipLaunchKernelGGL((combine_kernel<Y_BF16, X_BF16>), dim3(a.T), dim3(256), 0, s, a.y_slot, a.inv_perm, a.gates,
                       a.y_shared, a.x, a.w_shared_gate, a.residual, a.d, a.k, a.y, a.u_next, kRmsEps, a.slot_planes,
                       a.slot_plane_stride, a.shared_planes, a.shared_plane_stride);
}

// Chained stack: u[t] = h[t] / sqrt(mean_j h[t][j]^2 + eps), rounded to the layer dtype.  One workgroup per token;
// the sum of squares in a fixed order (per-thread strided fused multiply-adds, DPP tree, the four waves in order).
template <bool U_BF16>
__global__ void __launch_bounds__(256)
rmsnorm_kernel(const float* __restrict__ h, int d, float eps, void* __restrict__ u) {
    __shared__ float wave_part[4];
    const int t = blockIdx.x;
    const float* ht = h + (size_t)t * d;
    // d % 128 == 0 (checked at the boundary): 16-byte pieces, thread-strided
    float ss = 0.0f;
    for (int j = threadIdx.x * 4; j < d; j += 1024) {
        const f32x4_t v = *(const f32x4_t*)(ht + j);
#pragma unroll
        for (int i = 0; i < 4; ++i) ss = __builtin_fmaf(v[i], v[i], ss);
    }
    const float ws = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = ws;
    __syncthreads();
    const float total = ((wave_part[0] + wave_part[1]) + wave_part[2]) + wave_part[3];
    const float inv = 1.0f / sqrtf(total / (float)d + eps);
    for (int j = threadIdx.x * 4; j < d; j += 1024) {
        const f32x4_t v = *(const f32x4_t*)(ht + j);   // second read of the row: served by the cache
        store_normalised<U_BF16>(u, (size_t)t * d + j, v, inv);
    }
}

// h = x widened exactly to fp32 (the chained stack's hidden state starts as the input).
template <bool X_BF16>
__global__ void __launch_bounds__(256)
widen_kernel(const void* __restrict__ x, size_t n, float* __restrict__ h) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) h[i] = load_as_f32<X_BF16>(x, i);
}

hipError_t launch_rmsnorm(const float* h, int T, int d, float eps, void* u, bool u_bf16, hipStream_t s) {
    if (u_bf16) hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3(T), dim3(256), 0, s, h, d, eps, u);
    else hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3(T), dim3(256), 0, s, h, d, eps, u);
    return hipGetLastError();
}

hipError_t launch_widen(const void* x, bool x_bf16, size_t n, float* h, hipStream_t s) {
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (x_bf16) hipLaunchKernelGGL(widen_kernel<true>, dim3(blocks), dim3(256), 0, s, x, n, h);
    else hipLaunchKernelGGL(widen_kernel<false>, dim3(blocks), dim3(256), 0, s, x, n, h);
    return hipGetLastError();
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s) {
    if (a.y_bf16) { if (a.x_bf16) launch_combine_t<true, true>(a, s); else launch_combine_t<true, false>(a, s); }
    else          { if (a.x_bf16) launch_combine_t<false, true>(a, s); else launch_combine_t<false, false>(a, s); }
    return hipGetLastError();
}

}  // namespace lexi
