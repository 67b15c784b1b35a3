// Expert FFN kernels: grouped gate/up GEMM with fused SwiGLU, grouped down GEMM (paper Sec. 2: E_i(x), the part
// that holds nearly all parameters and FLOPs).  bf16 operands on MFMA with fp32 accumulation; a plain fp32 kernel
// covers fp32 layers.
//
// Orientation: the weight tile is the MFMA "A" operand (its 32 rows are features), the token tile is the "B"
// operand (its 32 columns are tokens).  In the 32x32 accumulator a lane then owns ONE token (column lane%32) and
// four groups of 4 consecutive features (rows 8g + 4*(lane/32) + 0..3), so the epilogue writes 8- or 16-byte
// runs along the feature axis, and SwiGLU pairs the gate and up accumulators register by register.
#include "kernels.hpp"

namespace lexi {

constexpr int BK = 64;         // K elements per LDS stage
constexpr int LDS_PAD = 8;     // bf16 elements of padding per LDS row (16 B): spreads the 16-byte operand reads over banks
constexpr int LDS_LD = BK + LDS_PAD;

struct TileInfo {
    int expert, row0, rows;
};

__device__ __forceinline__ bool fetch_tile(const int32_t* sched, const int32_t* sched_count, int tile, int M,
                                           int tile_tokens, TileInfo& ti) {
    if (sched != nullptr) {
        if (tile >= sched_count[0]) return false;
        const int32_t* s = sched + (size_t)tile * 4;
        ti.expert = s[0];
        ti.row0 = s[1];
        ti.rows = s[2];
        return true;
    }
    ti.expert = 0;
    ti.row0 = tile * tile_tokens;
    ti.rows = min(tile_tokens, M - ti.row0);
    return ti.rows > 0;
}

// ---------------------------------------------------------------------------------------------------------
// ffn_mfma_kernel<GATEUP>
//   Workgroup tile: 128 weight rows x 128 tokens, 4 waves as 2 (feature halves) x 2 (token halves); each wave owns
//   2 x 2 accumulator blocks of 32 x 32.  K advances in stages of 64 through double-buffered LDS.
//   GATEUP: weight rows 0..63 are gate rows f0..f0+63, rows 64..127 the matching up rows; the wave's two feature
//   blocks are (gate, up) of the same 32 features, so the epilogue is silu(gate)*up -> bf16 act[row][f].
//   DOWN:   weight rows are 128 consecutive output features; the epilogue stores fp32 out[row][j].
//   Token rows are gathered through row_token (no permuted copy of X is ever materialised).
// ---------------------------------------------------------------------------------------------------------
template <bool GATEUP>
__global__ void __launch_bounds__(256)
ffn_mfma_kernel(const bf16_t* __restrict__ in, const int32_t* __restrict__ row_token, const bf16_t* __restrict__ w0,
                const bf16_t* __restrict__ w1, int K, int features, int M, int tile_tokens,
                const int32_t* __restrict__ sched, const int32_t* __restrict__ sched_count, void* __restrict__ out) {
    constexpr int TT = 128;
    __shared__ __attribute__((aligned(16))) bf16_t lds_w[2][128 * LDS_LD];
    __shared__ __attribute__((aligned(16))) bf16_t lds_x[2][TT * LDS_LD];

    TileInfo ti;
    if (!fetch_tile(sched, sched_count, blockIdx.y, M, tile_tokens, ti)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wf = wave & 1, wt = wave >> 1;
    const int f0 = blockIdx.x * (GATEUP ? 64 : 128);  // first output feature of this workgroup

    // ---- global -> register staging: thread owns 16-byte chunk (tid % 8) of rows tid/8 + 32p ----
    const int chunk = tid & 7;
    const bf16_t* wsrc[4];
    const bf16_t* xsrc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = (tid >> 3) + 32 * p;
        if (GATEUP) {
            const bf16_t* base = (r < 64) ? w0 : w1;
            wsrc[p] = base + ((size_t)ti.expert * features + f0 + (r & 63)) * K + chunk * 8;
        } else {
            wsrc[p] = w0 + ((size_t)ti.expert * features + f0 + r) * K + chunk * 8;
        }
        const int rr = min(r, ti.rows - 1);  // rows past the group end re-read its last row; never stored
        const int src_row = row_token ? row_token[ti.row0 + rr] : ti.row0 + rr;
        xsrc[p] = in + (size_t)src_row * K + chunk * 8;
    }

    u32x4_t wreg[4], xreg[4];
    auto load_stage = [&](int kt) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            wreg[p] = *(const u32x4_t*)(wsrc[p] + kt * BK);
            xreg[p] = *(const u32x4_t*)(xsrc[p] + kt * BK);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = (tid >> 3) + 32 * p;
            *(u32x4_t*)(&lds_w[buf][r * LDS_LD + chunk * 8]) = wreg[p];
            *(u32x4_t*)(&lds_x[buf][r * LDS_LD + chunk * 8]) = xreg[p];
        }
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // LDS rows of this wave's feature blocks and token blocks
    int wrow[2], xrow[2];
#pragma unroll
    for (int fb = 0; fb < 2; ++fb) wrow[fb] = (GATEUP ? fb * 64 + wf * 32 : wf * 64 + fb * 32) + (lane & 31);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) xrow[tb] = wt * 64 + tb * 32 + (lane & 31);
    const int koff = (lane >> 5) * 8;

    const int nk = K / BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_stage(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t a[2], b[2];
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) a[fb] = *(const bf16x8_t*)(&lds_w[buf][wrow[fb] * LDS_LD + ks * 16 + koff]);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) b[tb] = *(const bf16x8_t*)(&lds_x[buf][xrow[tb] * LDS_LD + ks * 16 + koff]);
#pragma unroll
            for (int fb = 0; fb < 2; ++fb)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[fb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[fb], b[tb], acc[fb][tb], 0, 0, 0);
        }
        if (kt + 1 < nk) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue ----
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int r = wt * 64 + tb * 32 + (lane & 31);
        if (r >= ti.rows) continue;
        const size_t row = (size_t)(ti.row0 + r);
        if (GATEUP) {
            bf16_t* o = (bf16_t*)out + row * features + f0 + wf * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = silu(acc[0][tb][4 * g + i]) * acc[1][tb][4 * g + i];
                u32x2_t pk;
                pk[0] = pack_bf16x2(v[0], v[1]);
                pk[1] = pack_bf16x2(v[2], v[3]);
                *(u32x2_t*)(o + 8 * g) = pk;
            }
        } else {
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                float* o = (float*)out + row * features + f0 + wf * 64 + fb * 32 + (lane >> 5) * 4;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4_t v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = acc[fb][tb][4 * g + i];
                    *(f32x4_t*)(o + 8 * g) = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// fp32 layers: one thread per output element, fp32 fused multiply-add chain over K.  Plumbing-scale only.
// ---------------------------------------------------------------------------------------------------------
template <bool GATEUP>
__global__ void __launch_bounds__(256)
ffn_f32_kernel(const float* __restrict__ in, const int32_t* __restrict__ row_token, const float* __restrict__ w0,
               const float* __restrict__ w1, int K, int features, int M, int tile_tokens,
               const int32_t* __restrict__ sched, const int32_t* __restrict__ sched_count, float* __restrict__ out) {
    TileInfo ti;
    if (!fetch_tile(sched, sched_count, blockIdx.y, M, tile_tokens, ti)) return;
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= features) return;
    const float* wr0 = w0 + ((size_t)ti.expert * features + f) * K;
    const float* wr1 = GATEUP ? w1 + ((size_t)ti.expert * features + f) * K : nullptr;
    for (int r = 0; r < ti.rows; ++r) {
        const int src_row = row_token ? row_token[ti.row0 + r] : ti.row0 + r;
        const float* xr = in + (size_t)src_row * K;
        float a0 = 0.0f, a1 = 0.0f;
        for (int j = 0; j < K; ++j) {
            const float xv = xr[j];
            a0 = __builtin_fmaf(xv, wr0[j], a0);
            if (GATEUP) a1 = __builtin_fmaf(xv, wr1[j], a1);
        }
        out[(size_t)(ti.row0 + r) * features + f] = GATEUP ? silu(a0) * a1 : a0;
    }
}

template <bool GATEUP>
static hipError_t launch_ffn(const FfnArgs& a, hipStream_t s) {
    if (a.max_tiles <= 0) return hipSuccess;
    if (a.is_bf16) {
        const dim3 grid(a.features / (GATEUP ? 64 : 128), a.max_tiles);
        hipLaunchKernelGGL((ffn_mfma_kernel<GATEUP>), grid, dim3(256), 0, s, (const bf16_t*)a.in, a.row_token,
                           (const bf16_t*)a.w0, (const bf16_t*)a.w1, a.K, a.features, a.M, a.tile_tokens, a.sched,
                           a.sched_count, a.out);
    } else {
        const dim3 grid((a.features + 255) / 256, a.max_tiles);
        hipLaunchKernelGGL((ffn_f32_kernel<GATEUP>), grid, dim3(256), 0, s, (const float*)a.in, a.row_token,
                           (const float*)a.w0, (const float*)a.w1, a.K, a.features, a.M, a.tile_tokens, a.sched,
                           a.sched_count, (float*)a.out);
    }
    return hipGetLastError();
}

hipError_t launch_gateup(const FfnArgs& a, hipStream_t s) { return launch_ffn<true>(a, s); }
hipError_t launch_down(const FfnArgs& a, hipStream_t s) { return launch_ffn<false>(a, s); }

}  // namespace lexi
