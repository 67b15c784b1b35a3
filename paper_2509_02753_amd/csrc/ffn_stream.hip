// Expert FFN, weight-streaming schedule for decode-sized batches (a few rows per expert): the time goes into reading
// each touched expert's weights from HBM once, so the kernel is built around memory-level parallelism, not MFMA rate.
//
// A workgroup owns ONE unit of 16 output features of one token tile (gate/up: 16 gate rows + the 16 matching up
// rows) and splits the reduction dimension over its 4 waves.  A wave streams its quarter of the unit's packed
// 16 x 32 weight blocks -- 1 KB fully coalesced loads, many in flight -- and multiplies each against the tile's
// token blocks (16 tokens x 32 K, read straight from the token rows, which stay cache-resident) with
// v_mfma_f32_16x16x32_bf16.  The four partial accumulators are added in wave order through LDS (fixed order: same
// bits every run), then the epilogue of the tile schedule's kernel applies: silu(gate)*up -> bf16, or fp32 rows.
#include "ffn_common.hpp"

namespace lexi {

template <int N> struct IntTag { static constexpr int value = N; };

template <bool GATEUP>
__global__ void __launch_bounds__(256)
ffn_stream_kernel(const bf16_t* __restrict__ in, const int32_t* __restrict__ row_token, const bf16_t* __restrict__ w0,
                  const bf16_t* __restrict__ w1, int K, int features, int M, int tile_tokens,
                  const int32_t* __restrict__ sched, const int32_t* __restrict__ sched_count, void* __restrict__ out) {
    __shared__ __attribute__((aligned(16))) f32x4_t red[4][2][64];

    TileInfo ti;
    if (!fetch_tile(sched, sched_count, blockIdx.y, M, tile_tokens, ti)) return;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kq = lane >> 4;
    const int unit = blockIdx.x;  // output features 16*unit .. 16*unit+15
    const int nkb = K >> 5;
    const int kb0 = wave * nkb / 4, kb1 = (wave + 1) * nkb / 4;
    const size_t wbase = ((size_t)ti.expert * (features >> 4) + unit) * ((size_t)K * 16) + lane * 8;
    const bf16_t* a0 = w0 + wbase;
    const bf16_t* a1 = GATEUP ? w1 + wbase : nullptr;

    auto body = [&](auto ntb_tag) {
        constexpr int NTB = decltype(ntb_tag)::value;
        const bf16_t* xp[NTB];
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
            const int rr = min(tb * 16 + l16, ti.rows - 1);  // rows past the group end re-read its last row; never stored
            const int src_row = row_token ? row_token[ti.row0 + rr] : ti.row0 + rr;
            xp[tb] = in + (size_t)src_row * K + kq * 8;
        }
        f32x4_t accg[NTB], accu[NTB];
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
            accg[tb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
            accu[tb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
        }
        auto k_step = [&](int kb) {
            const bf16x8_t ag = *(const bf16x8_t*)(a0 + (size_t)kb * 512);
            bf16x8_t au;
            if (GATEUP) au = *(const bf16x8_t*)(a1 + (size_t)kb * 512);
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb) {
                const bf16x8_t b = *(const bf16x8_t*)(xp[tb] + kb * 32);
                accg[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag, b, accg[tb], 0, 0, 0);
                if (GATEUP) accu[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(au, b, accu[tb], 0, 0, 0);
            }
        };
        constexpr int UNROLL = NTB <= 2 ? 8 : 4;  // K blocks whose loads are in flight together
        int kb = kb0;
        for (; kb + UNROLL <= kb1; kb += UNROLL) {
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) k_step(kb + u);
        }
        for (; kb < kb1; ++kb) k_step(kb);
        // split-K reduction in wave order, one token block at a time; wave (tb % 4) finishes block tb
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) {
            red[wave][0][lane] = accg[tb];
            if (GATEUP) red[wave][1][lane] = accu[tb];
            __syncthreads();
            if (wave == (tb & 3)) {
                f32x4_t g = red[0][0][lane], u = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int w = 1; w < 4; ++w) g += red[w][0][lane];
                if (GATEUP) {
                    u = red[0][1][lane];
#pragma unroll
                    for (int w = 1; w < 4; ++w) u += red[w][1][lane];
                }
                const int r = tb * 16 + l16;  // lane owns token (lane % 16), features 4*(lane/16) + 0..3 of the unit
                if (r < ti.rows) {
                    const size_t row = (size_t)(ti.row0 + r);
                    if (GATEUP) {
                        u32x2_t pk;
                        pk[0] = pack_bf16x2(silu(g[0]) * u[0], silu(g[1]) * u[1]);
                        pk[1] = pack_bf16x2(silu(g[2]) * u[2], silu(g[3]) * u[3]);
                        *(u32x2_t*)((bf16_t*)out + row * features + unit * 16 + kq * 4) = pk;
                    } else {
                        *(f32x4_t*)((float*)out + row * features + unit * 16 + kq * 4) = g;
                    }
                }
            }
            __syncthreads();
        }
    };
    const int ntb = (ti.rows + 15) >> 4;
    if (ntb <= 1) body(IntTag<1>{});
    else if (ntb <= 2) body(IntTag<2>{});
    else if (ntb <= 4) body(IntTag<4>{});
    else body(IntTag<8>{});
}

template <bool GATEUP>
static hipError_t launch_stream(const FfnArgs& a, hipStream_t s) {
    if (a.max_tiles <= 0) return hipSuccess;
    const dim3 grid(a.features / 16, a.max_tiles);
    hipLaunchKernelGGL((ffn_stream_kernel<GATEUP>), grid, dim3(256), 0, s, (const bf16_t*)a.in, a.row_token,
                       (const bf16_t*)a.w0, (const bf16_t*)a.w1, a.K, a.features, a.M, a.tile_tokens, a.sched,
                       a.sched_count, a.out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// down_combine_kernel: for a handful of tokens the down projection's output rows (T*k x d fp32) are so small that
// writing them out and launching a second kernel to weight and add them costs more than the projection itself.  Here
// a workgroup of 16 waves owns 16 output features of ALL rows: it walks the experts that have rows (one tile each:
// an expert holds at most T <= 8 rows), several at a time -- the waves are dealt out as (experts per pass) x (parts
// of the reduction), the fewer experts the finer the split -- adds the parts in order through LDS, keeps the rows'
// 16 features in an LDS table, and finally forms y[t] = sum_s g[t][s] * row(t, s) in slot order, plus the shared
// expert's row, exactly as the combine kernel does.  Fixed orders throughout: same bits on every run.
// ---------------------------------------------------------------------------------------------------------
template <bool Y_BF16>
__global__ void __launch_bounds__(1024)
down_combine_kernel(const bf16_t* __restrict__ act, const bf16_t* __restrict__ w_down, int K, int d,
                    const int32_t* __restrict__ sched, const int32_t* __restrict__ sched_count,
                    const int32_t* __restrict__ inv_perm, const float* __restrict__ gates,
                    const float* __restrict__ y_shared, int T, int k, void* __restrict__ y) {
    __shared__ __attribute__((aligned(16))) f32x4_t red[16][64];
    __shared__ __attribute__((aligned(16))) f32x4_t ys[kFusedDownMaxRows][4];   // row -> the unit's 16 features

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kq = lane >> 4;
    const int unit = blockIdx.x;   // output features 16*unit .. 16*unit+15
    const int nkb = K >> 5;
    const int ntiles = sched_count[0];
    // combine: thread (t, q) owns features 16*unit + 4*q + 0..3 of token t; what it adds at the end that does not
    // depend on the projection is fetched now, under the weight stream
    const bool combiner = tid < T * 4;
    const int ct = tid >> 2, cq = tid & 3;
    const size_t cidx = (size_t)ct * d + unit * 16 + cq * 4;
    f32x4_t shared_row = {0.0f, 0.0f, 0.0f, 0.0f};
    if (combiner && y_shared != nullptr) shared_row = *(const f32x4_t*)(y_shared + cidx);
    constexpr int KPRE = 8;        // slots whose row index and gate are fetched ahead
    int32_t pre_row[KPRE];
    float pre_gate[KPRE];
#pragma unroll
    for (int s = 0; s < KPRE; ++s) {
        const bool have = combiner && s < k;
        pre_row[s] = have ? inv_perm[(size_t)ct * k + s] : 0;
        pre_gate[s] = have ? gates[(size_t)ct * k + s] : 0.0f;
    }
    // waves per expert: 16 for one expert, ..., 1 for nine or more (then 16 experts per pass)
    const int wpt = ntiles >= 9 ? 1 : ntiles >= 5 ? 2 : ntiles >= 3 ? 4 : ntiles == 2 ? 8 : 16;
    const int per_pass = 16 / wpt;
    const int sub = wave / wpt, kpart = wave - sub * wpt;

    for (int t0 = 0; t0 < ntiles; t0 += per_pass) {
        const int tile = t0 + sub;
        const bool live = tile < ntiles;   // wave-uniform
        int row0 = 0, rows = 0;
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (live) {
            const int32_t* sp = sched + (size_t)tile * kSchedStride;
            const int expert = sp[0];
            row0 = sp[1];
            rows = min(sp[2], 16);
            const int kb0 = kpart * nkb / wpt, kb1 = (kpart + 1) * nkb / wpt;
            const bf16_t* a0 = w_down + ((size_t)expert * (d >> 4) + unit) * ((size_t)K * 16) + lane * 8;
            // rows past the expert's end re-read its last row; their results are never used
            const bf16_t* xp = act + (size_t)(row0 + min(l16, rows - 1)) * K + kq * 8;
            auto k_step = [&](int kb) {
                const bf16x8_t ag = *(const bf16x8_t*)(a0 + (size_t)kb * 512);
                const bf16x8_t b = *(const bf16x8_t*)(xp + kb * 32);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag, b, acc, 0, 0, 0);
            };
            constexpr int UNROLL = 11;   // K blocks whose loads are in flight together
            int kb = kb0;
            for (; kb + UNROLL <= kb1; kb += UNROLL) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) k_step(kb + u);
            }
            for (; kb + 4 <= kb1; kb += 4) {
#pragma unroll
                for (int u = 0; u < 4; ++u) k_step(kb + u);
            }
            for (; kb < kb1; ++kb) k_step(kb);
        }
        red[wave][lane] = acc;
        __syncthreads();
        if (live && kpart == 0) {
            f32x4_t g = red[wave][lane];
            for (int p = 1; p < wpt; ++p) g += red[wave + p][lane];
            if (l16 < rows) ys[row0 + l16][kq] = g;   // lane owns row (lane % 16), features 4*(lane/16) + 0..3
        }
        __syncthreads();
    }

    if (!combiner) return;
    f32x4_t o = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < k; ++s) {   // slot order = rank order
        int32_t row;
        float g;
        if (s < KPRE) {
            row = pre_row[0]; g = pre_gate[0];
#pragma unroll
            for (int i = 1; i < KPRE; ++i)
                if (s == i) { row = pre_row[i]; g = pre_gate[i]; }
        } else {
            row = inv_perm[(size_t)ct * k + s];
            g = gates[(size_t)ct * k + s];
        }
        const f32x4_t v = ys[row][cq];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = __builtin_fmaf(g, v[i], o[i]);
    }
    if (y_shared != nullptr) {
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = __builtin_fmaf(1.0f, shared_row[i], o[i]);
    }
    if (Y_BF16) {
        u32x2_t pk;
        pk[0] = pack_bf16x2(o[0], o[1]);
        pk[1] = pack_bf16x2(o[2], o[3]);
        *(u32x2_t*)((bf16_t*)y + cidx) = pk;
    } else {
        *(f32x4_t*)((float*)y + cidx) = o;
    }
}

hipError_t launch_down_combine(const DownCombineArgs& a, hipStream_t s) {
    if (a.T < 1 || a.T > kFusedDownMaxT || a.T * a.k > kFusedDownMaxRows || a.d % 16 != 0 || a.F % 32 != 0)
        return hipErrorInvalidValue;
    const dim3 grid(a.d / 16);
    if (a.y_bf16)
        hipLaunchKernelGGL(down_combine_kernel<true>, grid, dim3(1024), 0, s, (const bf16_t*)a.act, (const bf16_t*)a.w_down,
                           a.F, a.d, a.sched, a.sched_count, a.inv_perm, a.gates, a.y_shared, a.T, a.k, a.y);
    else
        hipLaunchKernelGGL(down_combine_kernel<false>, grid, dim3(1024), 0, s, (const bf16_t*)a.act, (const bf16_t*)a.w_down,
                           a.F, a.d, a.sched, a.sched_count, a.inv_perm, a.gates, a.y_shared, a.T, a.k, a.y);
    return hipGetLastError();
}

hipError_t launch_gateup_stream(const FfnArgs& a, hipStream_t s) { return launch_stream<true>(a, s); }
hipError_t launch_down_stream(const FfnArgs& a, hipStream_t s) { return launch_stream<false>(a, s); }

}  // namespace lexi
