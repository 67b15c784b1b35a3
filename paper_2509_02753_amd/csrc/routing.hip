// Routing kernels: fp32 router GEMM + wave-level top-k + softmax over the selected, and the deterministic
// token-to-expert permutation (per-block histogram -> scan -> scatter).
//
// Paper Sec. 2: G(x) = Softmax(TopK[x * W_g]); k is a launch argument (Algorithm 1's UpdateTopk).
#include "kernels.hpp"

namespace lexi {

// ---------------------------------------------------------------------------------------------------------
// router_topk_kernel
//   One lane per expert (E <= 64), TM tokens per wave, WAVES waves per workgroup.
//   logits: the fixed order -- per 128-segment a chain of fused multiply-adds from +0, partials added in
//   ascending order, bias last.  The chain operand x[t][j] is wave-uniform (scalar loads), W[j][e] comes from an
//   LDS copy of the current segment shared by the waves of the workgroup.
//   top-k: k rounds of {wave maximum by DPP, ballot of the lanes that hold it, lowest set bit} -- the lowest
//   index among equal logits wins; comparisons are on floats, so +0 == -0.
//   Each selected (token, slot) also gets its rank among the workgroup's earlier assignments to the same expert
//   (tokens ascending), which is what makes the later scatter a stable counting sort without atomics.
// ---------------------------------------------------------------------------------------------------------
template <bool IS_BF16, int TM, int WAVES>
__global__ void __launch_bounds__(WAVES * 64)
router_topk_kernel(const void* __restrict__ x, const float* __restrict__ w_router, const float* __restrict__ bias,
                   int T, int d, int E, int k, int32_t* __restrict__ topk_idx, float* __restrict__ gates,
                   int32_t* __restrict__ local_rank, int32_t* __restrict__ blk_hist) {
    constexpr int TB = TM * WAVES;
    __shared__ float w_lds[kRouterSegment * 64];
    __shared__ int32_t wave_cnt[WAVES][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tok0 = blockIdx.x * TB + wave * TM;

    float total[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) total[m] = 0.0f;

    const int nseg = d / kRouterSegment;
    for (int seg = 0; seg < nseg; ++seg) {
        __syncthreads();
        for (int i = threadIdx.x; i < kRouterSegment * 64; i += WAVES * 64) {
            const int jj = i >> 6, e = i & 63;
            w_lds[i] = (e < E) ? w_router[(size_t)(seg * kRouterSegment + jj) * E + e] : 0.0f;
        }
        __syncthreads();

        float acc[TM];
#pragma unroll
        for (int m = 0; m < TM; ++m) acc[m] = 0.0f;

        for (int jj = 0; jj < kRouterSegment; jj += 8) {
            float w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = w_lds[(jj + i) * 64 + lane];
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                int t = tok0 + m;
                t = t < T ? t : T - 1;  // tail tokens recompute the last row; their results are never stored
                const size_t base = (size_t)t * d + seg * kRouterSegment + jj;
                float xv[8];
                if (IS_BF16) {
                    const u32x4_t p = *(const u32x4_t*)((const bf16_t*)x + base);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        xv[2 * i] = __uint_as_float(p[i] << 16);
                        xv[2 * i + 1] = __uint_as_float(p[i] & 0xFFFF0000u);
                    }
                } else {
                    const f32x4_t p0 = *(const f32x4_t*)((const float*)x + base);
                    const f32x4_t p1 = *(const f32x4_t*)((const float*)x + base + 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { xv[i] = p0[i]; xv[4 + i] = p1[i]; }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[m] = __builtin_fmaf(xv[i], w[i], acc[m]);
            }
        }
#pragma unroll
        for (int m = 0; m < TM; ++m) total[m] = (seg == 0) ? acc[m] : total[m] + acc[m];
    }

    const bool lane_valid = lane < E;
    if (bias != nullptr) {
        const float b = lane_valid ? bias[lane] : 0.0f;
#pragma unroll
        for (int m = 0; m < TM; ++m) total[m] = total[m] + b;
    }

    // ---- top-k, gates, per-wave ranks ----
    int32_t cnt = 0;           // lane e: assignments to expert e made so far by this wave
    int32_t sel[TM], rnk[TM];  // lane s (< k): expert, gate and rank-in-wave of slot s of token m
    float gte[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        float l = lane_valid ? total[m] : -INFINITY;
        bool taken = !lane_valid;
        const int32_t counted = (tok0 + m < T) ? 1 : 0;  // tail rows past T must not enter the histogram
        int32_t my_sel = 0, my_rank = 0;
        float my_val = -INFINITY;
        for (int s = 0; s < k; ++s) {
            const float cand = taken ? -INFINITY : l;
            const float mx = wave_max(cand);
            const uint64_t holders = __ballot(!taken && l == mx);
            const int e_star = __builtin_ctzll(holders);  // lowest index among equal logits
            const int32_t r = __builtin_amdgcn_readlane(cnt, e_star);
            if (lane == e_star) { taken = true; cnt += counted; }
            if (lane == s) { my_sel = e_star; my_val = mx; my_rank = r; }
        }
        // softmax over the selected logits; slot 0 holds the largest
        const float v0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_val), 0));
        const float ex = (lane < k) ? __expf(my_val - v0) : 0.0f;
        const float denom = wave_sum(ex);
        sel[m] = my_sel;
        rnk[m] = my_rank;
        gte[m] = ex / denom;
    }

    wave_cnt[wave][lane] = cnt;
    __syncthreads();
    if (wave == 0) {
        int32_t h = 0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) h += wave_cnt[w][lane];
        blk_hist[(size_t)blockIdx.x * 64 + lane] = h;
    }
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const int t = tok0 + m;
        if (t < T && lane < k) {
            int32_t before = 0;
            for (int w = 0; w < wave; ++w) before += wave_cnt[w][sel[m]];
            const size_t a = (size_t)t * k + lane;
            topk_idx[a] = sel[m];
            gates[a] = gte[m];
            local_rank[a] = before + rnk[m];
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// scan_kernel (one wave): per expert, exclusive prefix of the block histograms (in place), counts, offsets, and
// the token-tile schedule of the grouped GEMMs: tile i -> (expert, first row, rows).
// ---------------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64)
scan_kernel(int32_t* __restrict__ blk_hist, int nblk, int E, int tile_tokens, int32_t* __restrict__ counts,
            int32_t* __restrict__ offsets, int32_t* __restrict__ sched, int32_t* __restrict__ sched_count) {
    __shared__ int32_t s_cnt[64];
    __shared__ int32_t s_tiles[64];
    const int lane = threadIdx.x;
    int32_t running = 0;
    for (int b = 0; b < nblk; ++b) {
        const int32_t h = blk_hist[(size_t)b * 64 + lane];
        blk_hist[(size_t)b * 64 + lane] = running;
        running += h;
    }
    const int32_t ntile = (running + tile_tokens - 1) / tile_tokens;
    s_cnt[lane] = running;
    s_tiles[lane] = ntile;
    __syncthreads();
    int32_t off = 0, tile_base = 0;
    for (int e = 0; e < lane; ++e) { off += s_cnt[e]; tile_base += s_tiles[e]; }
    if (lane < E) {
        counts[lane] = running;
        offsets[lane] = off;
        for (int i = 0; i < ntile; ++i) {
            const int32_t rows = min(tile_tokens, running - i * tile_tokens);
            int32_t* s = sched + (size_t)(tile_base + i) * 4;
            s[0] = lane;                     // expert
            s[1] = off + i * tile_tokens;    // first permuted row
            s[2] = rows;                     // valid rows in this tile
            s[3] = 0;
        }
    }
    if (lane == 63) {
        // lanes >= E carry zero counts, so lane 63's exclusive sums plus its own are the totals
        offsets[E] = off + running;
        sched_count[0] = tile_base + ntile;
    }
}

// ---------------------------------------------------------------------------------------------------------
// permute_kernel: position of assignment a = offsets[e] + (assignments to e in earlier blocks) + rank in block.
// ---------------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
permute_kernel(const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ local_rank,
               const int32_t* __restrict__ blk_prefix, const int32_t* __restrict__ offsets, int A, int k,
               int tokens_per_block, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
               int32_t* __restrict__ row_token) {
    const int a = blockIdx.x * 256 + threadIdx.x;
    if (a >= A) return;
    const int e = topk_idx[a];
    const int t = a / k;
    const int blk = t / tokens_per_block;
    const int pos = offsets[e] + blk_prefix[(size_t)blk * 64 + e] + local_rank[a];
    perm[pos] = a;
    inv_perm[a] = pos;
    row_token[pos] = t;
}

// ---------------------------------------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------------------------------------
int router_tokens_per_block(int T) {
    if (T >= 256 * 32) return 32;
    if (T >= 256 * 16) return 16;
    return 8;
}

template <bool IS_BF16>
static hipError_t launch_router_t(const RoutingArgs& a, hipStream_t s) {
    const int tb = router_tokens_per_block(a.T);
    const int nblk = (a.T + tb - 1) / tb;
    if (tb == 32)
        hipLaunchKernelGGL((router_topk_kernel<IS_BF16, 8, 4>), dim3(nblk), dim3(256), 0, s, a.x, a.w_router, a.bias, a.T,
                           a.d, a.E, a.k, a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    else if (tb == 16)
        hipLaunchKernelGGL((router_topk_kernel<IS_BF16, 8, 2>), dim3(nblk), dim3(128), 0, s, a.x, a.w_router, a.bias, a.T,
                           a.d, a.E, a.k, a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    else
        hipLaunchKernelGGL((router_topk_kernel<IS_BF16, 8, 1>), dim3(nblk), dim3(64), 0, s, a.x, a.w_router, a.bias, a.T,
                           a.d, a.E, a.k, a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    return hipGetLastError();
}

hipError_t launch_routing(const RoutingArgs& a, hipStream_t s) {
    hipError_t err = a.is_bf16 ? launch_router_t<true>(a, s) : launch_router_t<false>(a, s);
    if (err != hipSuccess) return err;
    const int tb = router_tokens_per_block(a.T);
    const int nblk = (a.T + tb - 1) / tb;
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(64), 0, s, a.blk_hist, nblk, a.E, a.tile_tokens, a.counts, a.offsets,
                       a.sched, a.sched_count);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const int A = a.T * a.k;
    hipLaunchKernelGGL(permute_kernel, dim3((A + 255) / 256), dim3(256), 0, s, a.topk_idx, a.local_rank, a.blk_hist,
                       a.offsets, A, a.k, tb, a.perm, a.inv_perm, a.row_token);
    return hipGetLastError();
}

}  // namespace lexi
