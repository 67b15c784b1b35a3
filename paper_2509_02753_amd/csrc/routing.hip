// Routing kernels: fp32 router GEMM + wave-level top-k + softmax over the selected, and the deterministic
// token-to-expert permutation (per-block histogram -> scan -> scatter).
//
// Paper Sec. 2: G(x) = Softmax(TopK[x * W_g]); k is a launch argument (Algorithm 1's UpdateTopk).
#include "kernels.hpp"

namespace lexi {

// ---------------------------------------------------------------------------------------------------------
// The fp32 logit of (token t, expert e) has ONE defined evaluation order: d is cut into segments of 128; inside a
// segment the partial starts at +0 and takes one fused multiply-add per element, ascending; the partials are added
// in ascending segment order; the bias is added last.  The segment partials are independent chains, which is where
// the parallelism comes from: partial[seg][t][e] is produced by the two kernels below (a register-tiled one for
// prefill-sized T, a latency-oriented one for decode-sized T) and summed in order by topk_kernel.
// ---------------------------------------------------------------------------------------------------------

// router_partial_kernel: workgroup = 256 tokens x 64 experts x one segment, 8 waves.  A wave owns 64 tokens and one
// half of the experts; a lane owns an 8 (tokens) x 4 (experts) block of accumulators, so per j it reads 8 x-values and
// 4 w-values from LDS for 32 fused multiply-adds.  (Blocks of 8 x 8 with four waves leave one wave per SIMD, which
// measured 45 % of the plain-FMA rate; two waves per SIMD fill each other's issue gaps.)  x is staged through LDS
// transposed ([j][token], fp32) by the thread that owns the token row, W[j][e] row-major by the other four waves;
// the next 32-j stage is prefetched into registers while the current one is consumed.
template <bool IS_BF16>
__global__ void __launch_bounds__(512)
router_partial_kernel(const void* __restrict__ x, const float* __restrict__ w_router, int T, int d, int E,
                      float* __restrict__ partial) {
    constexpr int SJ = 32;                      // j per LDS stage
    constexpr int NSTAGE = kRouterSegment / SJ;
    __shared__ __attribute__((aligned(16))) float xs[4][SJ][64];
    __shared__ __attribute__((aligned(16))) float wsm[SJ][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tw = wave & 3, eh = wave >> 2;    // token quarter, expert half
    const int eg = lane & 7, tg = lane >> 3;
    const int seg = blockIdx.y;
    const int tok_base = blockIdx.x * 256;
    const bool x_loader = tid < 256;            // waves 0..3 stage x (one token row per thread), waves 4..7 stage W
    const int my_row = min(tok_base + (tid & 255), T - 1);  // rows past T re-read the last row; never stored
    const int j_seg = seg * kRouterSegment;

    u32x4_t xr[IS_BF16 ? 4 : 8];
    float wr[8];
    auto load_stage = [&](int st) {
        const int j0 = j_seg + st * SJ;
        if (x_loader) {
            if (IS_BF16) {
                const u32x4_t* p = (const u32x4_t*)((const bf16_t*)x + (size_t)my_row * d + j0);
#pragma unroll
                for (int i = 0; i < 4; ++i) xr[i] = p[i];
            } else {
                const u32x4_t* p = (const u32x4_t*)((const float*)x + (size_t)my_row * d + j0);
#pragma unroll
                for (int i = 0; i < 8; ++i) xr[i] = p[i];
            }
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int i = (tid - 256) + 256 * r, jj = i >> 6, e = i & 63;
                wr[r] = (e < E) ? w_router[(size_t)(j0 + jj) * E + e] : 0.0f;
            }
        }
    };
    auto store_stage = [&]() {
        if (x_loader) {
            if (IS_BF16) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        xs[wave][8 * i + 2 * c][lane] = __uint_as_float(xr[i][c] << 16);
                        xs[wave][8 * i + 2 * c + 1][lane] = __uint_as_float(xr[i][c] & 0xFFFF0000u);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int c = 0; c < 4; ++c) xs[wave][4 * i + c][lane] = __uint_as_float(xr[i][c]);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int i = (tid - 256) + 256 * r;
                wsm[i >> 6][i & 63] = wr[r];
            }
        }
    };

    float acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0f;

    load_stage(0);
    for (int st = 0; st < NSTAGE; ++st) {
        __syncthreads();
        store_stage();
        __syncthreads();
        if (st + 1 < NSTAGE) load_stage(st + 1);
#pragma unroll 4
        for (int jj = 0; jj < SJ; ++jj) {
            const f32x4_t x0 = *(const f32x4_t*)&xs[tw][jj][8 * tg];
            const f32x4_t x1 = *(const f32x4_t*)&xs[tw][jj][8 * tg + 4];
            const f32x4_t w0 = *(const f32x4_t*)&wsm[jj][32 * eh + 4 * eg];
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                const float xv = a < 4 ? x0[a & 3] : x1[a & 3];
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_fmaf(xv, w0[b], acc[a][b]);
            }
        }
    }

#pragma unroll
    for (int a = 0; a < 8; ++a) {
        const int t = tok_base + tw * 64 + 8 * tg + a;
        if (t < T) {
            float* o = partial + ((size_t)seg * T + t) * 64 + 32 * eh + 4 * eg;
            f32x4_t v0 = {acc[a][0], acc[a][1], acc[a][2], acc[a][3]};
            *(f32x4_t*)o = v0;
        }
    }
}

// router_partial_small_kernel: one wave = one segment x TW tokens, lane = expert.  The segment's 128 router weights
// of the lane's expert sit in registers (128 coalesced loads in flight at once); the token's x values are
// wave-uniform (scalar loads), so each token costs one 128-long chain of fused multiply-adds.
template <bool IS_BF16, int TW>
__global__ void __launch_bounds__(64)
router_partial_small_kernel(const void* __restrict__ x, const float* __restrict__ w_router, int T, int d, int E,
                            float* __restrict__ partial) {
    const int lane = threadIdx.x;
    const int seg = blockIdx.x;
    const int t0 = blockIdx.y * TW;
    const int j_seg = seg * kRouterSegment;
    float w[kRouterSegment];
    const float* wp = w_router + (size_t)j_seg * E + min(lane, E - 1);   // lanes >= E read a valid column; never used
#pragma unroll
    for (int jj = 0; jj < kRouterSegment; ++jj) w[jj] = wp[(size_t)jj * E];
    for (int m = 0; m < TW; ++m) {
        const int t = t0 + m;
        if (t >= T) break;
        float acc = 0.0f;
        if (IS_BF16) {
            const uint32_t* xp = (const uint32_t*)((const bf16_t*)x + (size_t)t * d + j_seg);
#pragma unroll
            for (int i = 0; i < kRouterSegment / 2; ++i) {
                const uint32_t p = xp[i];
                acc = __builtin_fmaf(__uint_as_float(p << 16), w[2 * i], acc);
                acc = __builtin_fmaf(__uint_as_float(p & 0xFFFF0000u), w[2 * i + 1], acc);
            }
        } else {
            const float* xp = (const float*)x + (size_t)t * d + j_seg;
#pragma unroll
            for (int i = 0; i < kRouterSegment; ++i) acc = __builtin_fmaf(xp[i], w[i], acc);
        }
        partial[((size_t)seg * T + t) * 64 + lane] = acc;
    }
}

// router_partial_narrow_kernel (prefill-sized T, exactly EW = 8 or 16 experts): with so few experts the 64-wide
// register tile above would spend most of its multiply-adds on padding.  Here a lane owns one token and all EW
// experts, a wave 64 tokens x one segment (the four waves of a workgroup take four neighbouring segments of the
// same tokens, 1 KB of each row together): the lane's 128 activations of the segment sit in registers (one
// contiguous 256-byte run of its row), the segment's weights are wave-uniform and come through scalar loads, so
// every instruction of the inner loop is a useful fused multiply-add.  Row stride of the partials: EW floats (no
// padding to 64 lanes).  (One segment per workgroup and 256 tokens instead measured 10 % slower.)
template <bool IS_BF16, int EW>
__global__ void __launch_bounds__(256)
router_partial_narrow_kernel(const void* __restrict__ x, const float* __restrict__ w_router, int T, int d,
                             float* __restrict__ partial) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int seg = blockIdx.y * 4 + wave;
    if (seg >= d / kRouterSegment) return;                 // (no barrier in this kernel)
    const int tok = blockIdx.x * 64 + lane;
    const int t = min(tok, T - 1);                         // rows past T re-read the last row; never stored
    const int j0 = seg * kRouterSegment;
    constexpr int NV = IS_BF16 ? kRouterSegment / 8 : kRouterSegment / 4;   // 16-byte pieces of the row segment
    u32x4_t xr[NV];
    const u32x4_t* xp = (const u32x4_t*)((const char*)x + ((size_t)t * d + j0) * (IS_BF16 ? 2 : 4));
#pragma unroll
    for (int i = 0; i < NV; ++i) xr[i] = xp[i];
    const float* __restrict__ wseg = w_router + (size_t)j0 * EW;   // [128][EW], wave-uniform
    float acc[EW];
#pragma unroll
    for (int e = 0; e < EW; ++e) acc[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (IS_BF16) {
                const float lo = __uint_as_float(xr[i][c] << 16), hi = __uint_as_float(xr[i][c] & 0xFFFF0000u);
                const int j = 8 * i + 2 * c;
#pragma unroll
                for (int e = 0; e < EW; ++e) acc[e] = __builtin_fmaf(lo, wseg[j * EW + e], acc[e]);
#pragma unroll
                for (int e = 0; e < EW; ++e) acc[e] = __builtin_fmaf(hi, wseg[(j + 1) * EW + e], acc[e]);
            } else {
                const float v = __uint_as_float(xr[i][c]);
                const int j = 4 * i + c;
#pragma unroll
                for (int e = 0; e < EW; ++e) acc[e] = __builtin_fmaf(v, wseg[j * EW + e], acc[e]);
            }
        }
    }
    if (tok < T) {
        float* o = partial + ((size_t)seg * T + tok) * EW;
#pragma unroll
        for (int e = 0; e < EW; e += 4) *(f32x4_t*)(o + e) = f32x4_t{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
    }
}

// ---------------------------------------------------------------------------------------------------------
// topk_kernel: one lane per expert (E <= 64), TM tokens per wave, WAVES waves per workgroup.
//   logit = ordered sum of the segment partials, then the bias.
//   top-k: k rounds of {wave maximum by DPP, ballot of the lanes that hold it, lowest set bit} -- the lowest
//   index among equal logits wins; comparisons are on floats, so +0 == -0.
//   gates: softmax over the k selected logits.
//   Each selected (token, slot) also gets its rank among the workgroup's earlier assignments to the same expert
//   (tokens ascending), which is what makes the later scatter a stable counting sort without atomics.
// ---------------------------------------------------------------------------------------------------------
template <int TM, int WAVES>
__global__ void __launch_bounds__(WAVES * 64)
topk_kernel(const float* __restrict__ partial, int pstride, const float* __restrict__ bias, int T, int nseg, int E, int k,
            int32_t* __restrict__ topk_idx, float* __restrict__ gates, int32_t* __restrict__ local_rank,
            int32_t* __restrict__ blk_hist) {
    constexpr int TB = TM * WAVES;
    __shared__ int32_t wave_cnt[WAVES][64];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tok0 = blockIdx.x * TB + wave * TM;
    const int tok_end = T;

    // a row of partials holds `pstride` floats (64, or the expert count of the narrow partial kernel); lanes past it
    // hold no expert and load nothing
    const bool has_col = lane < pstride;
    float total[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const int t = min(tok0 + m, T - 1);
        total[m] = has_col ? partial[(size_t)t * pstride + lane] : 0.0f;
    }
    // ordered sum of the remaining partials; the loads of CH segments are issued together (the adds stay in order)
    constexpr int CH = 8;
    for (int sg0 = 1; sg0 < nseg; sg0 += CH) {
        float tmp[CH][TM];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int sg = min(sg0 + c, nseg - 1);
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                const int t = min(tok0 + m, T - 1);
                tmp[c][m] = has_col ? partial[((size_t)sg * T + t) * pstride + lane] : 0.0f;
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if (sg0 + c < nseg) {
#pragma unroll
                for (int m = 0; m < TM; ++m) total[m] = total[m] + tmp[c][m];
            }
        }
    }
    const bool lane_valid = lane < E;
    if (bias != nullptr) {
        const float b = lane_valid ? bias[lane] : 0.0f;
#pragma unroll
        for (int m = 0; m < TM; ++m) total[m] = total[m] + b;
    }
    // Inputs are finite by contract.  A NaN logit (one NaN or Inf activation is enough) compares unequal to every
    // maximum, which would leave the ballot below empty and the expert index undefined; it ranks as -inf instead, so
    // every round selects a valid expert (all-NaN row: experts 0..k-1) and the token's gates and output come out NaN.
#pragma unroll
    for (int m = 0; m < TM; ++m) total[m] = (total[m] == total[m]) ? total[m] : -INFINITY;

    // ---- top-k: slot-major, token-minor, so the TM independent reduction chains of one round overlap ----
    uint32_t taken = 0;        // lane e: bit m set once token m has selected expert e
    int32_t sel[TM];           // lane s (< k): expert in slot s of token m
    float val[TM];             // lane s (< k): its logit
#pragma unroll
    for (int m = 0; m < TM; ++m) { sel[m] = 0; val[m] = -INFINITY; }
    for (int s = 0; s < k; ++s) {
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            if (tok0 + m < tok_end) {  // wave-uniform: rows past the wave's range are skipped
                const bool open = lane_valid && !((taken >> m) & 1u);
                const float mx = wave_max(open ? total[m] : -INFINITY);
                const uint64_t holders = __ballot(open && total[m] == mx);
                const int e_star = __builtin_ctzll(holders);  // lowest index among equal logits
                if (lane == e_star) taken |= 1u << m;
                if (lane == s) { sel[m] = e_star; val[m] = mx; }
            }
        }
    }
    // ---- gates: softmax over the selected logits; slot 0 holds the largest ----
    float gte[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const float v0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(val[m]), 0));
        const float ex = (lane < k) ? __expf(val[m] - v0) : 0.0f;
        gte[m] = ex / wave_sum(ex);
    }
    // ---- rank of each assignment among this wave's earlier assignments to the same expert (tokens ascending):
    //      lane e counts its own expert's hits in token order, the slot lanes fetch theirs with one permute ----
    int32_t cnt = 0;
    int32_t rnk[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        rnk[m] = __builtin_amdgcn_ds_bpermute(sel[m] << 2, cnt);
        cnt += (int32_t)((taken >> m) & 1u);
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
// scan_kernel (one workgroup of 16 waves): per expert, exclusive prefix of the block histograms (in place),
// counts, offsets, and the token-tile schedule of the grouped GEMMs: 8 ints per tile (expert, the expert's first
// row and row count, index of the tile inside the expert, tiles of the expert).
// Wave w scans its contiguous chunk of blocks, the chunk totals are combined through LDS.
// ---------------------------------------------------------------------------------------------------------
// With FUSE_PERMUTE (decode-sized batches) the same workgroup then scatters the assignments (the body of
// permute_kernel), which saves a launch on the latency-bound path.
template <bool FUSE_PERMUTE>
__global__ void __launch_bounds__(1024)
scan_kernel(int32_t* __restrict__ blk_hist, int nblk, int E, int tile_tokens, int32_t* __restrict__ counts,
            int32_t* __restrict__ offsets, int32_t* __restrict__ sched, int32_t* __restrict__ sched_count,
            const int32_t* __restrict__ topk_idx, const int32_t* __restrict__ local_rank, int A, int k,
            int tokens_per_block, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
            int32_t* __restrict__ row_token) {
    __shared__ int32_t chunk_tot[16][64];
    __shared__ int32_t s_cnt[64];
    __shared__ int32_t s_tiles[64];
    __shared__ int32_t s_off[64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = (nblk + 15) / 16;
    const int b0 = wave * chunk, b1 = min(nblk, b0 + chunk);
    // the chunk's histograms are loaded eight at a time (independent loads in flight), then prefixed in order
    int32_t running = 0;
    for (int b = b0; b < b1; b += 8) {
        int32_t h[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) h[u] = blk_hist[(size_t)min(b + u, b1 - 1) * 64 + lane];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (b + u < b1) {
                blk_hist[(size_t)(b + u) * 64 + lane] = running;
                running += h[u];
            }
        }
    }
    chunk_tot[wave][lane] = running;
    __syncthreads();
    int32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int32_t c = chunk_tot[w][lane];
        base += (w < wave) ? c : 0;
        total += c;
    }
    if (base != 0) {
        for (int b = b0; b < b1; b += 8) {
            int32_t h[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) h[u] = blk_hist[(size_t)min(b + u, b1 - 1) * 64 + lane];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (b + u < b1) blk_hist[(size_t)(b + u) * 64 + lane] = h[u] + base;
        }
    }
    const int32_t ntile = (total + tile_tokens - 1) / tile_tokens;
    if (wave == 0) {
        s_cnt[lane] = total;
        s_tiles[lane] = ntile;
    }
    __syncthreads();
    if (wave == 0) {
        int32_t off = 0, tile_base = 0;
        for (int e = 0; e < lane; ++e) { off += s_cnt[e]; tile_base += s_tiles[e]; }
        s_off[lane] = off;
        if (lane < E) {
            counts[lane] = total;
            offsets[lane] = off;
            for (int i = 0; i < ntile; ++i) {
                int32_t* s = sched + (size_t)(tile_base + i) * 8;
                s[0] = lane;      // expert
                s[1] = off;       // first permuted row of the expert
                s[2] = total;     // rows of the expert
                s[3] = i;         // index of the tile inside its expert
                s[4] = ntile;     // tiles of the expert
            }
        }
        if (lane == 63) {
            // lanes >= E carry zero counts, so lane 63's exclusive sums plus its own are the totals
            offsets[E] = off + total;
            sched_count[0] = tile_base + ntile;
        }
    }
    if (!FUSE_PERMUTE) return;
    __syncthreads();   // s_off, and this workgroup's own writes to blk_hist, are visible to all its waves from here
    for (int a = threadIdx.x; a < A; a += 1024) {
        const int e = topk_idx[a];
        const int t = a / k;
        const int blk = t / tokens_per_block;
        const int pos = s_off[e] + blk_hist[(size_t)blk * 64 + e] + local_rank[a];
        perm[pos] = a;
        inv_perm[a] = pos;
        row_token[pos] = t;
    }
}

// ---------------------------------------------------------------------------------------------------------
// topk_scan_kernel (decode-sized batches, T <= kFusedTailMaxT): ONE workgroup of 16 waves does everything after the
// segment partials -- the top-k and gates of every token (one token per wave per pass, tokens ascending), the
// per-expert counts, offsets and tile schedule, and the scatter.  With all tokens in one workgroup the stable
// counting sort needs no block histograms in memory: an assignment's position is offsets[e] + (assignments to e by
// earlier tokens), kept in LDS.  Saves two dependent launches on the latency-bound path.
// ---------------------------------------------------------------------------------------------------------
constexpr int kFusedTailMaxT = 16;
constexpr int kFusedTailMaxA = kFusedTailMaxT * 64;   // assignments (k <= E <= 64)

__global__ void __launch_bounds__(1024)
topk_scan_kernel(const float* __restrict__ partial, const float* __restrict__ bias, int T, int nseg, int E, int k,
                 int tile_tokens, int32_t* __restrict__ topk_idx, float* __restrict__ gates,
                 int32_t* __restrict__ counts, int32_t* __restrict__ offsets, int32_t* __restrict__ sched,
                 int32_t* __restrict__ sched_count, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                 int32_t* __restrict__ row_token) {
    __shared__ int32_t wave_hit[16][64];        // this pass: 1 if the wave's token selected expert e
    __shared__ int32_t s_seen[64];              // assignments to expert e by the tokens of earlier passes
    __shared__ int32_t s_tiles[64];
    __shared__ int32_t s_off[64];
    __shared__ uint8_t s_e[kFusedTailMaxA];     // expert of assignment a
    __shared__ int16_t s_rank[kFusedTailMaxA];  // assignments to that expert by earlier tokens
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool lane_valid = lane < E;
    if (wave == 0) s_seen[lane] = 0;
    const float b = (bias != nullptr && lane_valid) ? bias[lane] : 0.0f;
    __syncthreads();
    for (int t0 = 0; t0 < T; t0 += 16) {
        const int t = t0 + wave;
        const bool live = t < T;                // wave-uniform
        int32_t sel = 0;
        bool hit = false;
        if (live) {
            // logit = ordered sum of the segment partials, then the bias (same order as topk_kernel)
            float total = partial[(size_t)t * 64 + lane];
            for (int sg0 = 1; sg0 < nseg; sg0 += 8) {
                float tmp[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) tmp[c] = partial[((size_t)min(sg0 + c, nseg - 1) * T + t) * 64 + lane];
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    if (sg0 + c < nseg) total = total + tmp[c];
            }
            if (bias != nullptr) total = total + b;
            total = (total == total) ? total : -INFINITY;   // a NaN logit ranks last (see topk_kernel)
            float val = -INFINITY;
            for (int s = 0; s < k; ++s) {
                const bool open = lane_valid && !hit;
                const float mx = wave_max(open ? total : -INFINITY);
                const uint64_t holders = __ballot(open && total == mx);
                const int e_star = __builtin_ctzll(holders);   // lowest index among equal logits
                if (lane == e_star) hit = true;
                if (lane == s) { sel = e_star; val = mx; }
            }
            const float v0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(val), 0));
            const float ex = (lane < k) ? __expf(val - v0) : 0.0f;
            const float g = ex / wave_sum(ex);
            if (lane < k) {
                const size_t a = (size_t)t * k + lane;
                topk_idx[a] = sel;
                gates[a] = g;
                s_e[a] = (uint8_t)sel;
            }
        }
        wave_hit[wave][lane] = hit ? 1 : 0;
        __syncthreads();
        if (live && lane < k) {
            int32_t before = s_seen[sel];
            for (int w = 0; w < wave; ++w) before += wave_hit[w][sel];
            s_rank[t * k + lane] = (int16_t)before;
        }
        __syncthreads();
        if (wave == 0) {
            int32_t h = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) h += wave_hit[w][lane];
            s_seen[lane] += h;
        }
        __syncthreads();
    }
    if (wave == 0) {
        const int32_t total = s_seen[lane];
        const int32_t ntile = (total + tile_tokens - 1) / tile_tokens;
        s_tiles[lane] = ntile;
        __builtin_amdgcn_s_waitcnt(0);          // wave 0 reads what its own lanes wrote: order the LDS accesses
        __builtin_amdgcn_wave_barrier();
        int32_t off = 0, tile_base = 0;
        for (int e = 0; e < lane; ++e) { off += s_seen[e]; tile_base += s_tiles[e]; }
        s_off[lane] = off;
        if (lane < E) {
            counts[lane] = total;
            offsets[lane] = off;
            for (int i = 0; i < ntile; ++i) {
                int32_t* sp = sched + (size_t)(tile_base + i) * 8;
                sp[0] = lane; sp[1] = off; sp[2] = total; sp[3] = i; sp[4] = ntile;
            }
        }
        if (lane == 63) {
            offsets[E] = off + total;
            sched_count[0] = tile_base + ntile;
        }
    }
    __syncthreads();
    const int A = T * k;
    for (int a = threadIdx.x; a < A; a += 1024) {
        const int pos = s_off[s_e[a]] + s_rank[a];
        perm[pos] = a;
        inv_perm[a] = pos;
        row_token[pos] = a / k;
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
constexpr int kTinyRouterMaxT = 128;    // at or below: one token per wave in the partial and top-k kernels
constexpr int kSmallRouterMaxT = 1024;  // at or below this many tokens the latency-oriented partial kernel runs

int router_tokens_per_block(int T) { return T >= 2048 ? 16 : 8; }

// Row stride of the segment partials: the narrow kernel (prefill-sized T, exactly 8 or 16 experts) packs them.
static int partial_stride(const RoutingArgs& a) {
    return (a.T > kSmallRouterMaxT && (a.E == 8 || a.E == 16)) ? a.E : 64;
}

template <bool IS_BF16>
static hipError_t launch_partials(const RoutingArgs& a, hipStream_t s) {
    const int nseg = a.d / kRouterSegment;
    if (partial_stride(a) != 64) {
        const dim3 grid((a.T + 63) / 64, (nseg + 3) / 4);
        if (a.E == 8)
            hipLaunchKernelGGL((router_partial_narrow_kernel<IS_BF16, 8>), grid, dim3(256), 0, s, a.x, a.w_router, a.T, a.d, a.partial);
        else
            hipLaunchKernelGGL((router_partial_narrow_kernel<IS_BF16, 16>), grid, dim3(256), 0, s, a.x, a.w_router, a.T, a.d, a.partial);
        return hipGetLastError();
    }
    if (a.T <= kTinyRouterMaxT) {
        // a handful of tokens: one token per wave, so the chains of different tokens run on different CUs
        hipLaunchKernelGGL((router_partial_small_kernel<IS_BF16, 1>), dim3(nseg, a.T), dim3(64), 0, s, a.x, a.w_router,
                           a.T, a.d, a.E, a.partial);
    } else if (a.T <= kSmallRouterMaxT) {
        constexpr int TW = 4;
        hipLaunchKernelGGL((router_partial_small_kernel<IS_BF16, TW>), dim3(nseg, (a.T + TW - 1) / TW), dim3(64), 0, s,
                           a.x, a.w_router, a.T, a.d, a.E, a.partial);
    } else {
        hipLaunchKernelGGL((router_partial_kernel<IS_BF16>), dim3((a.T + 255) / 256, nseg), dim3(512), 0, s, a.x,
                           a.w_router, a.T, a.d, a.E, a.partial);
    }
    return hipGetLastError();
}

hipError_t launch_routing(const RoutingArgs& a, hipStream_t s) {
    hipError_t err = a.is_bf16 ? launch_partials<true>(a, s) : launch_partials<false>(a, s);
    if (err != hipSuccess) return err;
    const int nseg = a.d / kRouterSegment;
    if (a.T <= kFusedTailMaxT) {
        hipLaunchKernelGGL(topk_scan_kernel, dim3(1), dim3(1024), 0, s, a.partial, a.bias, a.T, nseg, a.E, a.k,
                           a.tile_tokens, a.topk_idx, a.gates, a.counts, a.offsets, a.sched, a.sched_count, a.perm,
                           a.inv_perm, a.row_token);
        return hipGetLastError();
    }
    const int tb = router_tokens_per_block(a.T);
    const int nblk = (a.T + tb - 1) / tb;
    const int ps = partial_stride(a);
    if (tb == 16)
        hipLaunchKernelGGL((topk_kernel<4, 4>), dim3(nblk), dim3(256), 0, s, a.partial, ps, a.bias, a.T, nseg, a.E, a.k,
                           a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    else if (a.T <= kTinyRouterMaxT)
        hipLaunchKernelGGL((topk_kernel<1, 8>), dim3(nblk), dim3(512), 0, s, a.partial, ps, a.bias, a.T, nseg, a.E, a.k,
                           a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    else
        hipLaunchKernelGGL((topk_kernel<8, 1>), dim3(nblk), dim3(64), 0, s, a.partial, ps, a.bias, a.T, nseg, a.E, a.k,
                           a.topk_idx, a.gates, a.local_rank, a.blk_hist);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    const int A = a.T * a.k;
    if (a.T <= kSmallRouterMaxT) {   // decode-sized: the scan's workgroup scatters the assignments itself
        hipLaunchKernelGGL(scan_kernel<true>, dim3(1), dim3(1024), 0, s, a.blk_hist, nblk, a.E, a.tile_tokens, a.counts,
                           a.offsets, a.sched, a.sched_count, a.topk_idx, a.local_rank, A, a.k, tb, a.perm, a.inv_perm,
                           a.row_token);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(scan_kernel<false>, dim3(1), dim3(1024), 0, s, a.blk_hist, nblk, a.E, a.tile_tokens, a.counts,
                       a.offsets, a.sched, a.sched_count, a.topk_idx, a.local_rank, A, a.k, tb, a.perm, a.inv_perm,
                       a.row_token);
    if ((err = hipGetLastError()) != hipSuccess) return err;
    hipLaunchKernelGGL(permute_kernel, dim3((A + 255) / 256), dim3(256), 0, s, a.topk_idx, a.local_rank, a.blk_hist,
                       a.offsets, A, a.k, tb, a.perm, a.inv_perm, a.row_token);
    return hipGetLastError();
}

}  // namespace lexi
