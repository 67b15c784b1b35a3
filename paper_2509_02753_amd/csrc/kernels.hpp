// Internal launch interface between the C ABI (api.hip) and the kernel translation units.
#pragma once
#include "common.hpp"

namespace lexi {

struct RoutingArgs {
    const void* x;            // [T][d]
    bool is_bf16;
    const float* w_router;    // [d][E]
    const float* bias;        // [E] or null
    int T, d, E, k;
    int tile_tokens;          // token-tile height the grouped GEMM schedule is built for
    float* partial;           // [d/128][T][64] segment partials of the logits
    int32_t* topk_idx;        // [T*k]
    float* gates;             // [T*k]
    int32_t* local_rank;      // [T*k]  rank of the assignment inside its router block, per expert
    int32_t* blk_hist;        // [nblk][64] histogram, turned into per-expert block prefixes by the scan
    int32_t* counts;          // [E]
    int32_t* offsets;         // [E+1]
    int32_t* perm;            // [T*k]
    int32_t* inv_perm;        // [T*k]
    int32_t* row_token;       // [T*k]  permuted row -> token
    int32_t* sched;           // [max_tiles][8]  (expert, its first row, its rows, tile index in it, its tiles, 0, 0, 0)
    int32_t* sched_count;     // [1]
};

int router_tokens_per_block(int T);
hipError_t launch_routing(const RoutingArgs& a, hipStream_t s);

// One grouped (or dense) GEMM of the expert FFN.
//   GATE/UP:  act[r][f] = silu(in[tok(r)] . Wg[e][f]) * (in[tok(r)] . Wu[e][f])      K = d, features = F
//   DOWN:     out[r][j] = act[r] . Wd[e][j]                                           K = F, features = d
// rows r are the permuted assignment rows (grouped: tile schedule from the scan) or plain token rows (dense, sched
// == null: one group of M rows, expert 0).
struct FfnArgs {
    bool is_bf16;
    bool streaming;            // few rows per expert: use the weight-streaming (HBM-bound) schedule
    const void* in;            // row-major [*][K]
    const int32_t* row_token;  // gather map row -> input row, or null (identity)
    int in_rows;               // rows of `in` when row_token is given (bound of the gather)
    const void* w0;            // gate (GATE/UP) or down weights, [E] packed matrices of [features][K]
    const void* w1;            // up weights or null
    int K;                     // reduction length
    int features;              // F (gate/up) or d (down)
    int M;                     // total rows (dense mode bound / grid sizing)
    int max_tiles;             // upper bound on the number of token tiles
    int tile_tokens;           // must equal the value the schedule was built with
    const int32_t* sched;      // null = dense
    const int32_t* sched_count;
    void* out;                 // GATE/UP: act [rows][F] (layer dtype);  DOWN: [rows][d] fp32
    // DOWN on the tile schedule only:
    int ksplit;                // 1, or 2: the reduction is cut in two halves, half h writes plane h of `out`
    size_t plane_stride;       // elements between the planes of `out`
    const int32_t* scatter;    // null, or row -> output row: rows are stored at out[scatter[row]] (ksplit must be 1)
    bool out_bf16;             // with scatter: `out` is bf16 (nearest-even rounding of the fp32 result) instead of fp32
};

hipError_t launch_gateup(const FfnArgs& a, hipStream_t s);
hipError_t launch_down(const FfnArgs& a, hipStream_t s);

// row-major [n_mat][R][K] -> packed expert-weight layout (R % 16 == 0, K % 32 == 0)
hipError_t launch_pack(const void* src, void* dst, int64_t n_mat, int R, int K, bool is_bf16, hipStream_t s);

struct CombineArgs {
    const float* y_slot;       // [T*k][d] fp32, permuted rows; `slot_planes` planes, `slot_plane_stride` elements apart,
                               // that are added (plane order) before the gate is applied
    int slot_planes;
    size_t slot_plane_stride;
    const int32_t* inv_perm;   // [T*k]
    const float* gates;        // [T*k]
    const float* y_shared;     // [T][d] fp32 or null; `shared_planes` planes likewise
    int shared_planes;
    size_t shared_plane_stride;
    const void* x;             // [T][d] layer input (only read for a sigmoid-gated shared expert)
    const void* w_shared_gate; // [d] or null (ungated: coefficient 1)
    bool x_bf16;
    int T, d, k;
    const float* residual;     // [T][d] fp32 added to the result (chained stack), or null; may alias y
    void* y;                   // [T][d]
    bool y_bf16;
    void* u_next;              // chained stack: [T][d] layer dtype, the next block's normalised input, or null
};
hipError_t launch_combine(const CombineArgs& a, hipStream_t s);

// Down projection and combine of a decode-sized batch in one launch (bf16 layers, T <= kFusedDownMaxT, T*k <=
// kFusedDownMaxRows, shared expert absent or ungated): y[t] = sum_s gates[t][s] * (act[row(t, s)] . W_down[e]) in slot
// order, then the shared expert's row.
constexpr int kFusedDownMaxT = 8;      // beyond these the separate launches measured faster (more experts with rows than
constexpr int kFusedDownMaxRows = 64;  // the d/16 workgroups of the fused launch can stream at full rate)
struct DownCombineArgs {
    const void* act;           // [T*k][F] bf16, permuted rows
    const void* w_down;        // [E] packed matrices of [d][F]
    int F, d, T, k;
    const int32_t* sched;      // tile schedule (one tile per expert with rows)
    const int32_t* sched_count;
    const int32_t* inv_perm;   // [T*k]
    const float* gates;        // [T*k]
    const float* y_shared;     // [T][d] fp32 or null (added with coefficient 1)
    void* y;                   // [T][d]
    bool y_bf16;
};
hipError_t launch_down_combine(const DownCombineArgs& a, hipStream_t s);

// chained stack: normalised MoE input u (layer dtype) from the fp32 hidden state h; h = widened x
constexpr float kRmsEps = 1e-6f;
hipError_t launch_rmsnorm(const float* h, int T, int d, float eps, void* u, bool u_bf16, hipStream_t s);
hipError_t launch_widen(const void* x, bool x_bf16, size_t n, float* h, hipStream_t s);

// Stage-1 profiling: squared-difference reduction over the slot rows of one baseline pass.
constexpr int kProfileMaxK = 64;
struct ProfileKList {          // passed to the kernel by value
    int32_t n;
    int32_t k[kProfileMaxK];
};
struct ProfileArgs {
    const float* y_slot;       // [T*k_base][d] fp32, permuted rows
    const int32_t* inv_perm;   // [T*k_base]
    const float* gates;        // [T*k_base] baseline gates
    int T, d, k_base;
    ProfileKList klist;
    float* part;               // [n][T] per-token squared norms
    float* delta;              // [n]
};
hipError_t launch_profile(const ProfileArgs& a, hipStream_t s);

}  // namespace lexi
