// Expert FFN kernels: grouped gate/up GEMM with fused SwiGLU, grouped down GEMM (paper Sec. 2: E_i(x), the part
// that holds nearly all parameters and FLOPs).  bf16 operands on MFMA with fp32 accumulation; a plain fp32 kernel
// covers fp32 layers.
//
// Orientation: the weight block is the MFMA "A" operand (its 16 rows are features), the token block is the "B"
// operand (its 16 columns are tokens).  In the 16x16 accumulator a lane then owns ONE token (column lane%16) and
// 4 consecutive features (rows 4*(lane/16) + 0..3), so the epilogue writes 8- or 16-byte runs along the feature
// axis, and SwiGLU pairs the gate and up accumulators register by register.
#include "ffn_common.hpp"

namespace lexi {

// ---------------------------------------------------------------------------------------------------------
// ffn_mfma_kernel<GATEUP>
//   Workgroup = 4 waves; token tile = 128 rows shared by all waves through double-buffered LDS; each wave owns its
//   own 64 weight rows (4 feature blocks of 16) against all 128 tokens (8 token blocks): 32 accumulator blocks of
//   16 x 16 (v_mfma_f32_16x16x32_bf16), i.e. a 256 x 128 workgroup tile in at most 256 registers per lane, so two
//   workgroups share a CU and one's prologue/epilogue overlaps the other's MFMA loop.  Weight rows are not shared between waves
//   and are stored in the packed layout, so their MFMA operand fragments go straight from global memory to
//   registers as fully coalesced 1 KB wave loads; only the token tile passes through LDS (8 fragment reads per 32 MFMAs).
//   GATEUP: a wave's blocks 0,1 are gate rows g0..g0+31 and blocks 2,3 the matching up rows, so the epilogue is
//   silu(gate)*up -> bf16 act[row][f]; the workgroup covers 128 hidden features.
//   DOWN:   a wave's blocks are 64 consecutive output features; the epilogue stores fp32 out[row][j].  Options: the
//           reduction cut in two halves handled by two workgroups that write two planes of `out` (more, shorter work
//           items when a launch would otherwise leave most CUs idle in its last round; the consumer adds the planes);
//           rows stored at out[scatter[row]] in the caller's dtype (layers with one active expert: no combine pass).
//   Token rows are gathered through row_token (no permuted copy of X is ever materialised).
//   Waves whose feature range lies past `features` (ragged last workgroup column) only help staging the tokens.
// ---------------------------------------------------------------------------------------------------------
template <int S> struct StageTag { static constexpr int value = S; };

template <bool GATEUP>
__global__ void __launch_bounds__(256, 2)
ffn_mfma_kernel(const bf16_t* __restrict__ in, const int32_t* __restrict__ row_token, const bf16_t* __restrict__ w0,
                const bf16_t* __restrict__ w1, int K, int features, int M, int tile_tokens,
                const int32_t* __restrict__ sched, const int32_t* __restrict__ sched_count, void* __restrict__ out,
                int ksplit, size_t plane_stride, const int32_t* __restrict__ scatter, int out_bf16) {
    constexpr int TT = 128, TB = TT / 16, WB = 4, KS = BK / 32;
    __shared__ __attribute__((aligned(16))) bf16_t lds_x[2][TT * LDS_LD];

    TileInfo ti;
    int cb, part = 0;
    if (!fetch_item(sched, sched_count, (features + (GATEUP ? 127 : 255)) / (GATEUP ? 128 : 256), M, tile_tokens, ti, cb,
                    GATEUP ? 1 : ksplit, &part))
        return;
    // DOWN with a split reduction: this workgroup covers K-steps [part * nk, (part + 1) * nk) and writes plane `part`
    const int nk = GATEUP ? K / BK : K / BK / ksplit;
    const uint32_t kstep0 = GATEUP ? 0u : (uint32_t)(part * nk);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_f0 = cb * (GATEUP ? 128 : 256) + wave * (GATEUP ? 32 : 64);  // first output feature
    const bool active = wave_f0 < features;
    const int l16 = lane & 15, kq = lane >> 4;
    const int koff = kq * 8;

    // ---- weight fragments: feature block fb of this wave is 16 packed rows; one K-step of 32 is one 1 KB block, a
    //      lane reads its 16 bytes at lane*16; successive K-steps are 1 KB apart.  The block-row origins are
    //      wave-uniform and live in scalar registers, the lane part is one 32-bit offset (a packed 16-row slab is
    //      32*K bytes, far below 4 GiB): 64-bit per-lane pointers would push the kernel over its 256 registers.
    const char* abase[WB];
#pragma unroll
    for (int fb = 0; fb < WB; ++fb) {
        int row;
        const bf16_t* base = w0;
        if (GATEUP) {
            row = wave_f0 + 16 * (fb & 1);
            if (fb >= 2) base = w1;
        } else {
            row = wave_f0 + 16 * fb;
        }
        row = active ? row : 0;
        abase[fb] = (const char*)(base + ((size_t)ti.expert * (features >> 4) + (row >> 4)) * ((size_t)K * 16)) +
                    (size_t)kstep0 * (KS * 1024);
    }
    const uint32_t alane = lane * 16;

    // ---- token tile staging: thread owns 16-byte chunk (tid % 8) of rows tid/8 + 32p ----
    const int chunk = tid & 7;
    uint32_t xoff[4];   // byte offsets from `in` (the launcher rejects inputs of 4 GiB or more)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int r = (tid >> 3) + 32 * p;
        const int rr = min(r, ti.rows - 1);  // rows past the group end re-read its last row; never stored
        const int src_row = row_token ? row_token[ti.row0 + rr] : ti.row0 + rr;
        xoff[p] = (uint32_t)(((size_t)src_row * K + (size_t)kstep0 * BK + chunk * 8) * 2);
    }
    u32x4_t xreg[4];
    auto load_x = [&](int kt) {
#pragma unroll
        for (int p = 0; p < 4; ++p) xreg[p] = *(const u32x4_t*)((const char*)in + (xoff[p] + (uint32_t)kt * (BK * 2)));
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *(u32x4_t*)(&lds_x[buf][((tid >> 3) + 32 * p) * LDS_LD + chunk * 8]) = xreg[p];
    };

    f32x4_t acc[WB][TB];
#pragma unroll
    for (int a = 0; a < WB; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.0f;

    bf16x8_t areg[WB][KS];
    load_x(0);
#pragma unroll
    for (int fb = 0; fb < WB; ++fb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) areg[fb][ks] = *(const bf16x8_t*)(abase[fb] + (alane + (uint32_t)ks * 1024u));
    store_x(0);
    __syncthreads();

    // The K loop, specialised on the number of 16-token blocks the tile really holds: the last tile of an expert's
    // group (and every tile of a decode-sized batch) skips the MFMAs of token blocks that would only hold padding.
    auto k_loop = [&](auto ntb_tag) {
        constexpr int NTB = decltype(ntb_tag)::value;
        for (int kt = 0; kt < nk; ++kt) {
            const int buf = kt & 1;
            const int kn = min(kt + 1, nk - 1);  // the last stage re-fetches itself: branch-free, in bounds, unused
            load_x(kn);
            __builtin_amdgcn_sched_barrier(0);  // keep the token-tile loads at the top: they are consumed after the MFMAs
            // (waves of a ragged last column run the same loop on weight row 0 instead of branching around it)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8_t b[NTB];
#pragma unroll
                for (int tb = 0; tb < NTB; ++tb)
                    b[tb] = *(const bf16x8_t*)(&lds_x[buf][(tb * 16 + l16) * LDS_LD + ks * 32 + koff]);
#pragma unroll
                for (int fb = 0; fb < WB; ++fb)
#pragma unroll
                    for (int tb = 0; tb < NTB; ++tb)
                        acc[fb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(areg[fb][ks], b[tb], acc[fb][tb], 0, 0, 0);
#pragma unroll
                for (int fb = 0; fb < WB; ++fb) areg[fb][ks] = *(const bf16x8_t*)(abase[fb] + (alane + (uint32_t)(kn * KS + ks) * 1024u));
                __builtin_amdgcn_sched_barrier(0);  // refill each fragment right after its last use, one k-step at a time
            }
            store_x(buf ^ 1);
            __syncthreads();
        }
    };
    switch ((ti.rows + 15) >> 4) {
        case 1: k_loop(StageTag<1>{}); break;
        case 2: k_loop(StageTag<2>{}); break;
        case 3: k_loop(StageTag<3>{}); break;
        case 4: k_loop(StageTag<4>{}); break;
        case 5: k_loop(StageTag<5>{}); break;
        case 6: k_loop(StageTag<6>{}); break;
        case 7: k_loop(StageTag<7>{}); break;
        default: k_loop(StageTag<8>{}); break;
    }
    // ---- epilogue: in a 16 x 16 accumulator block a lane owns token (lane % 16) and features 4*(lane/16) + 0..3
    if (GATEUP) {
        // The workgroup's 128 tokens x 128 features of silu(gate)*up are transposed through LDS (the token-tile
        // buffers are free now), so that the global stores are whole 256-byte rows instead of 8-byte pieces.
        // Row stride 272 B: the 8-byte writes of a half-wave (16 tokens x 2 lane groups) then fall on 64 distinct banks.
        constexpr int ELD = 136;   // bf16 elements per staged row
        static_assert(TT * ELD <= 2 * TT * LDS_LD, "the staged output tile must fit the token-tile buffers");
        bf16_t* stage = &lds_x[0][0];
        __syncthreads();           // every wave is done reading the token tile
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (tb * 16 >= ti.rows) break;
#pragma unroll
            for (int fb = 0; fb < 2; ++fb) {
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = silu(acc[fb][tb][i]) * acc[fb + 2][tb][i];
                u32x2_t pk;
                pk[0] = pack_bf16x2(v[0], v[1]);
                pk[1] = pack_bf16x2(v[2], v[3]);
                *(u32x2_t*)(&stage[(tb * 16 + l16) * ELD + wave * 32 + fb * 16 + kq * 4]) = pk;
            }
        }
        __syncthreads();
        const int c16 = tid & 15;                       // 16-byte chunk of the 256-byte row
        const int f = cb * 128 + c16 * 8;               // first of its 8 features
        if (f < features) {                             // (ragged last column block: features is a multiple of 64)
#pragma unroll
            for (int p = 0; p < TT / 16; ++p) {
                const int r = (tid >> 4) + 16 * p;
                if (r < ti.rows)
                    *(u32x4_t*)((bf16_t*)out + (size_t)(ti.row0 + r) * features + f) = *(const u32x4_t*)(&stage[r * ELD + c16 * 8]);
            }
        }
    } else {
        // (a register transpose to 64-byte runs per lane was measured slower than these 16-byte pieces, which L2 merges)
        if (!active) return;
        if (scatter != nullptr) {
            // one active expert per token (gate exactly 1): the row is the layer's output row of its token
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const int r = tb * 16 + l16;
                if (r >= ti.rows) continue;
                const size_t o = (size_t)scatter[ti.row0 + r] * features + wave_f0 + kq * 4;
#pragma unroll
                for (int fb = 0; fb < WB; ++fb) {
                    if (out_bf16) {
                        u32x2_t pk;
                        pk[0] = pack_bf16x2(acc[fb][tb][0], acc[fb][tb][1]);
                        pk[1] = pack_bf16x2(acc[fb][tb][2], acc[fb][tb][3]);
                        *(u32x2_t*)((bf16_t*)out + o + 16 * fb) = pk;
                    } else {
                        *(f32x4_t*)((float*)out + o + 16 * fb) = acc[fb][tb];
                    }
                }
            }
            return;
        }
        float* plane = (float*)out + (size_t)part * plane_stride;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const int r = tb * 16 + l16;
            if (r >= ti.rows) continue;
            float* o = plane + (size_t)(ti.row0 + r) * features + wave_f0 + kq * 4;
#pragma unroll
            for (int fb = 0; fb < WB; ++fb) *(f32x4_t*)(o + 16 * fb) = acc[fb][tb];
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
    const float* wr0 = w0 + (size_t)ti.expert * features * K;
    const float* wr1 = GATEUP ? w1 + (size_t)ti.expert * features * K : nullptr;
    for (int r = 0; r < ti.rows; ++r) {
        const int src_row = row_token ? row_token[ti.row0 + r] : ti.row0 + r;
        const float* xr = in + (size_t)src_row * K;
        float a0 = 0.0f, a1 = 0.0f;
        for (int j = 0; j < K; ++j) {
            const float xv = xr[j];
            const size_t wi = packed_index(f, j, K);
            a0 = __builtin_fmaf(xv, wr0[wi], a0);
            if (GATEUP) a1 = __builtin_fmaf(xv, wr1[wi], a1);
        }
        out[(size_t)(ti.row0 + r) * features + f] = GATEUP ? silu(a0) * a1 : a0;
    }
}

// pack_kernel: row-major [n_mat][R][K] -> packed layout, one 16-byte (bf16) or 32-byte (fp32) run per thread.
template <typename VEC>
__global__ void __launch_bounds__(256)
pack_kernel(const VEC* __restrict__ src, VEC* __restrict__ dst, int R, int K, size_t runs_total) {
    const size_t run = (size_t)blockIdx.x * 256 + threadIdx.x;  // index of the destination run
    if (run >= runs_total) return;
    const size_t runs_per_mat = (size_t)R * (K >> 3);
    const size_t mat = run / runs_per_mat;
    const size_t in_mat = run % runs_per_mat;
    const int i = (int)(in_mat & 15), q = (int)((in_mat >> 4) & 3);
    const size_t blk = in_mat >> 6;
    const int kb = (int)(blk % (size_t)(K >> 5)), rb = (int)(blk / (size_t)(K >> 5));
    const int r = rb * 16 + i, k = kb * 32 + q * 8;
    dst[run] = src[mat * runs_per_mat + ((size_t)r * K + k) / 8];
}

hipError_t launch_pack(const void* src, void* dst, int64_t n_mat, int R, int K, bool is_bf16, hipStream_t s) {
    const size_t runs = (size_t)n_mat * R * (K >> 3);
    if (runs == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((runs + 255) / 256);
    if (is_bf16) {
        hipLaunchKernelGGL(pack_kernel<u32x4_t>, dim3(blocks), dim3(256), 0, s, (const u32x4_t*)src, (u32x4_t*)dst, R, K, runs);
    } else {
        typedef __attribute__((ext_vector_type(8))) uint32_t u32x8_t;
        hipLaunchKernelGGL(pack_kernel<u32x8_t>, dim3(blocks), dim3(256), 0, s, (const u32x8_t*)src, (u32x8_t*)dst, R, K, runs);
    }
    return hipGetLastError();
}

template <bool GATEUP>
static hipError_t launch_ffn(const FfnArgs& a, hipStream_t s) {
    if (a.max_tiles <= 0) return hipSuccess;
    if ((a.ksplit > 1 || a.scatter != nullptr) && !(a.is_bf16 && !a.streaming && !GATEUP))
        return hipErrorInvalidValue;   // split reduction and scattered rows exist on the bf16 tile schedule's DOWN only
    if (a.is_bf16 && a.streaming) return GATEUP ? launch_gateup_stream(a, s) : launch_down_stream(a, s);
    if (a.is_bf16) {
        // the tile kernel addresses its input rows with 32-bit byte offsets
        const size_t in_rows = a.row_token ? (size_t)a.in_rows : (size_t)a.M;
        if (in_rows * (size_t)a.K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
        const int ncb = (a.features + (GATEUP ? 127 : 255)) / (GATEUP ? 128 : 256);
        const int ksplit = GATEUP ? 1 : (a.ksplit > 1 ? a.ksplit : 1);
        if (ksplit > 1 && ((a.K / BK) % ksplit != 0 || a.scatter != nullptr)) return hipErrorInvalidValue;
        const dim3 grid(xcd_grid(ncb, a.max_tiles, ksplit));
        hipLaunchKernelGGL((ffn_mfma_kernel<GATEUP>), grid, dim3(256), 0, s, (const bf16_t*)a.in, a.row_token,
                           (const bf16_t*)a.w0, (const bf16_t*)a.w1, a.K, a.features, a.M, a.tile_tokens, a.sched,
                           a.sched_count, a.out, ksplit, a.plane_stride, GATEUP ? nullptr : a.scatter, a.out_bf16 ? 1 : 0);
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
