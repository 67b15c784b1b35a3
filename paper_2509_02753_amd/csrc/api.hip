// C ABI of the library: argument validation, workspace slicing and the per-layer launch sequence.
// Nothing here allocates, synchronises or copies to the host; every launch goes to the caller's stream.
#include "../../include/lexi_moe.h"
#include "kernels.hpp"
#include <mutex>

namespace {

using namespace lexi;

constexpr int kTileTokens = 128;  // token-tile height of the grouped GEMM kernels
constexpr int kStreamRowsPerExpert = 2;   // mean rows per expert at or below which the routed FFN streams weights
constexpr int kStreamDownMaxItems = 256;   // (token tiles x column blocks) at or below which the routed down GEMM streams
constexpr int kStreamDenseRows = 64;      // token count at or below which the shared expert streams weights

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Split of the down GEMM's reduction dimension on the tile schedule.  A launch runs (token tiles x column blocks of
// 256 features) work items on 512 workgroup slots (two per CU).  When a launch with a long reduction cannot fill
// those slots even once, cutting the reduction in two gives twice as many items of half the length; the halves land
// in two planes of the output that the consumer adds.  Eligible: at least 32 K-steps of 64, an even number of them.
// Taken when the expected number of items (full tiles plus half a ragged tile per expert; the real number is only
// known on the device) is at most half the slots and the time saved outweighs writing and re-reading the second
// plane.  (For launches of several rounds, e.g. 1100 items of 14336, the split measured no gain in the down GEMM and
// cost the combine a second plane, so it is not taken there.)
constexpr int kWorkgroupSlots = 512;
inline bool ksplit_eligible(int K) { return K / 64 >= 32 && (K / 64) % 2 == 0; }
int choose_ksplit(int64_t rows, int groups, int K, int features, bool is_bf16) {
    if (!is_bf16 || !ksplit_eligible(K) || rows <= 0) return 1;
    const double ragged = groups > 1 ? 0.5 * (double)(groups < rows ? groups : rows) : (rows % kTileTokens ? 0.5 : 0.0);
    const double items = ((double)(rows / kTileTokens) + ragged) * ((features + 255) / 256);
    if (items > kWorkgroupSlots / 2) return 1;
    const double t_item = (2.0 * kTileTokens * 256.0 * K) / 3.9e12;           // one item at what one CU sustains
    const double t_plane = 2.0 * (double)rows * features * 4.0 / 5.0e12;      // second plane: written once, read once
    return 0.5 * t_item > 1.5 * t_plane ? 2 : 1;
}

// The shared expert depends on x only, not on the routing, so for decode-sized batches (where its kernels are short
// and latency-bound) it runs on a side stream that forks from the caller's stream at the start of the layer and joins
// it again in front of the combine.  One side stream and one event pair per device, created on first use and kept
// until the process ends; the caller sees plain stream semantics (and a capture of the caller's stream picks the
// side stream up through the events).
constexpr int kSideStreamMaxT = 1024;
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool tried = false, ok = false;
};
constexpr int kMaxDevices = 16;
SideStream g_side[kMaxDevices];
std::mutex g_side_mutex, g_side_enqueue_mutex;

SideStream* side_stream() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_side_mutex);
    SideStream& ss = g_side[dev];
    if (!ss.tried) {
        ss.tried = true;
        ss.ok = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
                hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess;
    }
    return ss.ok ? &ss : nullptr;   // no side stream: the shared expert simply stays on the caller's stream
}

// Scratch of lexi_moe_layer_forward_static: the workspace of one decode-sized layer call, held in the library's own
// device image so that the call needs no allocation and no workspace argument.  Every GPU the library runs on holds
// its own copy until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// device address is looked up once per device and used from then on.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
void* g_static_scratch_ptr[kMaxDevices] = {};
std::mutex g_static_scratch_mutex;

// Device address of the current device's copy of the scratch array, or null.
void* static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (g_static_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess) return nullptr;
        g_static_scratch_ptr[dev] = p;
    }
    return g_static_scratch_ptr[dev];
}

// Walks the workspace once; with base == nullptr it only measures.
struct Carver {
    char* base;
    size_t used = 0;
    explicit Carver(void* b) : base((char*)b) {}
    template <typename T>
    T* take(size_t count) {
        used = align_up(used, 256);
        T* p = base ? (T*)(base + used) : nullptr;
        used += count * sizeof(T);
        return p;
    }
};

struct Workspace {
    int32_t *topk_idx, *local_rank, *blk_hist, *counts, *offsets, *perm, *inv_perm, *row_token, *sched, *sched_count;
    float *gates, *partial, *y_slot, *y_shared;
    void *act, *act_shared, *u;
    int max_tiles;
    int slot_planes = 1, shared_planes = 1;   // planes of y_slot / y_shared the last launches wrote
    bool direct = false;                      // the routed down GEMM wrote the layer's output itself
    bool fused = false;                       // the caller launches down + combine as one kernel (run_routed stopped after gate/up)
    size_t bytes;
};

Workspace carve(const lexi_layer_t& ly, int T, int k, void* base) {
    Workspace w{};
    Carver c(base);
    const size_t A = (size_t)T * k;
    const size_t es = ly.dtype == LEXI_BF16 ? 2 : 4;
    const size_t nblk = ((size_t)T + 7) / 8;  // router blocks never hold fewer than 8 tokens
    // every expert with rows has one ragged tile at most, the rest are full
    w.max_tiles = (int)(A / kTileTokens) + (int)(A < (size_t)ly.E ? A : (size_t)ly.E);
    // chained stack: the normalised MoE input.  First, so that its place does not depend on the layer or on k: a
    // block's combine writes the next block's input there.
    w.u = c.take<char>((size_t)T * ly.d * es);
    w.partial = c.take<float>((size_t)(ly.d / 128) * T * 64);
    w.topk_idx = c.take<int32_t>(A);
    w.gates = c.take<float>(A);
    w.local_rank = c.take<int32_t>(A);
    w.blk_hist = c.take<int32_t>(nblk * 64);
    w.counts = c.take<int32_t>(64);
    w.offsets = c.take<int32_t>(68);
    w.perm = c.take<int32_t>(A);
    w.inv_perm = c.take<int32_t>(A);
    w.row_token = c.take<int32_t>(A);
    w.sched = c.take<int32_t>((size_t)w.max_tiles * 8);
    w.sched_count = c.take<int32_t>(4);
    w.act = c.take<char>(A * ly.F * es);
    // two planes wherever the down GEMM may split its reduction (independent of T and k, so that the size asked for
    // at (T_max, k_max) covers every smaller call)
    const bool bf = ly.dtype == LEXI_BF16;
    w.y_slot = c.take<float>(A * ly.d * ((bf && ksplit_eligible(ly.F)) ? 2 : 1));
    if (ly.F_shared > 0) {
        w.act_shared = c.take<char>((size_t)T * ly.F_shared * es);
        w.y_shared = c.take<float>((size_t)T * ly.d * ((bf && ksplit_eligible(ly.F_shared)) ? 2 : 1));
    }
    w.bytes = align_up(c.used, 256);
    return w;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

lexi_status check_layer(const lexi_layer_t* ly) {
    if (ly == nullptr) return LEXI_ERR_NULL;
    if (ly->dtype != LEXI_F32 && ly->dtype != LEXI_BF16) return LEXI_ERR_DTYPE;
    if (ly->shared_kind < LEXI_SHARED_NONE || ly->shared_kind > LEXI_SHARED_SIGMOID) return LEXI_ERR_DTYPE;
    if (ly->E < 1 || ly->E > 64) return LEXI_ERR_SHAPE;
    if (ly->d < 128 || ly->d % 128 != 0) return LEXI_ERR_SHAPE;
    if (ly->F < 64 || ly->F % 64 != 0) return LEXI_ERR_SHAPE;
    if (ly->F_shared < 0 || ly->F_shared % 64 != 0) return LEXI_ERR_SHAPE;
    if ((ly->F_shared > 0) != (ly->shared_kind != LEXI_SHARED_NONE)) return LEXI_ERR_SHAPE;
    if (!ly->w_router || !ly->w_gate || !ly->w_up || !ly->w_down) return LEXI_ERR_NULL;
    if (ly->F_shared > 0 && (!ly->ws_gate || !ly->ws_up || !ly->ws_down)) return LEXI_ERR_NULL;
    if (ly->shared_kind == LEXI_SHARED_SIGMOID && !ly->w_shared_gate) return LEXI_ERR_NULL;
    const void* ptrs[] = {ly->w_router, ly->router_bias, ly->w_gate, ly->w_up, ly->w_down,
                          ly->ws_gate, ly->ws_up, ly->ws_down, ly->w_shared_gate};
    for (const void* p : ptrs)
        if (p && misaligned(p)) return LEXI_ERR_ALIGN;
    return LEXI_OK;
}

// Limits on (T, k) that every entry point running the routed path shares.
lexi_status check_sizes(const lexi_layer_t* ly, int32_t T, int32_t k) {
    if (T < 0) return LEXI_ERR_SHAPE;
    if (k < 1 || k > ly->E) return LEXI_ERR_BAD_K;
    if ((int64_t)T * k >= (1 << 24)) return LEXI_ERR_SHAPE;
    // the tile kernels address their input rows with 32-bit byte offsets
    const uint64_t es = ly->dtype == LEXI_BF16 ? 2 : 4, lim = (uint64_t)1 << 32;
    if ((uint64_t)T * ly->d * es >= lim || (uint64_t)T * k * ly->F * es >= lim || (uint64_t)T * ly->F_shared * es >= lim)
        return LEXI_ERR_SHAPE;
    return LEXI_OK;
}

lexi_status check_call(const lexi_layer_t* ly, const void* x, const void* y, int32_t y_dtype, int32_t T, int32_t k,
                       const void* workspace, size_t workspace_bytes, const lexi_routing_out_t* dbg) {
    lexi_status st = check_layer(ly);
    if (st != LEXI_OK) return st;
    if (y_dtype != LEXI_F32 && y_dtype != LEXI_BF16) return LEXI_ERR_DTYPE;
    st = check_sizes(ly, T, k);
    if (st != LEXI_OK) return st;
    if (T == 0) return LEXI_OK;
    if (!x || !y || !workspace) return LEXI_ERR_NULL;
    if (misaligned(x) || misaligned(y) || misaligned(workspace)) return LEXI_ERR_ALIGN;
    if (dbg) {
        const void* ptrs[] = {dbg->topk_idx, dbg->gates, dbg->counts, dbg->offsets, dbg->perm, dbg->inv_perm, dbg->moe_input};
        for (const void* p : ptrs)
            if (p && misaligned(p)) return LEXI_ERR_ALIGN;
    }
    if (workspace_bytes < carve(*ly, T, k, nullptr).bytes) return LEXI_ERR_WORKSPACE;
    return LEXI_OK;
}

// Routing and the routed expert GEMMs of one layer at top-k = k: fills the routing arrays, act and y_slot of `w`.
// `allow_split`: the down GEMM may write two planes of y_slot (w.slot_planes tells).  `direct_y` != null (k == 1, nothing
// else to add): the down GEMM stores the output rows straight into the layer's output (w.direct tells whether it did).
// Launch plan of the down GEMMs of one call (also what lexi_moe_down_plan reports).
struct DownPlan {
    bool routed_streams, shared_streams;   // weight-streaming schedule instead of the tile schedule
    int routed_ksplit, shared_ksplit;      // parts of the reduction on the tile schedule (1 or 2)
    bool routed_direct;                    // with k == 1 and nothing to add: rows stored straight into y
    bool routed_fused;                     // a handful of tokens: down projection and combine in one launch
};
DownPlan plan_down(const lexi_layer_t& ly, int32_t T, int32_t k, bool allow_split, bool allow_direct) {
    DownPlan p{};
    const bool bf = ly.dtype == LEXI_BF16;
    const int64_t A = (int64_t)T * k;
    const int max_tiles = (int)(A / kTileTokens) + (int)(A < ly.E ? A : ly.E);
    const bool stream_routed = A <= (int64_t)kStreamRowsPerExpert * ly.E;
    // the down projection has few column blocks (d / 256): with few token tiles as well the tile schedule would leave
    // most CUs idle, so it streams too (16-feature units, K split over the waves)
    p.routed_streams = stream_routed || (int64_t)max_tiles * ((ly.d + 255) / 256) <= kStreamDownMaxItems;
    p.shared_streams = T <= kStreamDenseRows;
    p.routed_ksplit = p.shared_ksplit = 1;
    const bool tile_routed = bf && !p.routed_streams;
    p.routed_direct = tile_routed && allow_direct && k == 1 && ly.F_shared == 0;
    // (allow_direct: the caller wants nothing but y -- no slot rows, no residual, no normalised copy)
    p.routed_fused = bf && p.routed_streams && allow_direct && T <= kFusedDownMaxT && A <= kFusedDownMaxRows &&
                     ly.shared_kind != LEXI_SHARED_SIGMOID;
    if (tile_routed && allow_split && !p.routed_direct) p.routed_ksplit = choose_ksplit(A, ly.E, ly.F, ly.d, bf);
    if (ly.F_shared > 0 && bf && !p.shared_streams) p.shared_ksplit = choose_ksplit(T, 1, ly.F_shared, ly.d, bf);
    return p;
}

lexi_status run_routed(const lexi_layer_t& ly, const void* x, int32_t T, int32_t k, Workspace& w, hipStream_t s,
                       const lexi_stage_events_t* events, bool allow_split = true, void* direct_y = nullptr,
                       bool direct_bf16 = false) {
    auto mark = [&](int i) {
        if (events && events->ev[i]) (void)hipEventRecord((hipEvent_t)events->ev[i], s);
    };
    const bool bf = ly.dtype == LEXI_BF16;
    RoutingArgs r{};
    r.x = x; r.is_bf16 = bf; r.w_router = ly.w_router; r.bias = ly.router_bias;
    r.T = T; r.d = ly.d; r.E = ly.E; r.k = k; r.tile_tokens = kTileTokens;
    r.partial = w.partial; r.topk_idx = w.topk_idx; r.gates = w.gates; r.local_rank = w.local_rank; r.blk_hist = w.blk_hist;
    r.counts = w.counts; r.offsets = w.offsets; r.perm = w.perm; r.inv_perm = w.inv_perm; r.row_token = w.row_token;
    r.sched = w.sched; r.sched_count = w.sched_count;
    if (launch_routing(r, s) != hipSuccess) return LEXI_ERR_LAUNCH;
    mark(1);

    // few rows per expert (decode): the weight-streaming schedule; otherwise the MFMA tile schedule
    const bool stream_routed = (int64_t)T * k <= (int64_t)kStreamRowsPerExpert * ly.E;
    FfnArgs g{};
    g.streaming = stream_routed;
    g.is_bf16 = bf; g.in = x; g.row_token = w.row_token; g.in_rows = T; g.w0 = ly.w_gate; g.w1 = ly.w_up; g.K = ly.d;
    g.features = ly.F; g.M = T * k; g.max_tiles = w.max_tiles; g.tile_tokens = kTileTokens; g.sched = w.sched;
    g.sched_count = w.sched_count; g.out = w.act;
    if (launch_gateup(g, s) != hipSuccess) return LEXI_ERR_LAUNCH;
    mark(2);

    FfnArgs dn{};
    dn.is_bf16 = bf; dn.in = w.act; dn.row_token = nullptr; dn.w0 = ly.w_down; dn.w1 = nullptr; dn.K = ly.F;
    dn.features = ly.d; dn.M = T * k; dn.max_tiles = w.max_tiles; dn.tile_tokens = kTileTokens; dn.sched = w.sched;
    dn.sched_count = w.sched_count; dn.out = w.y_slot;
    const DownPlan plan = plan_down(ly, T, k, allow_split, direct_y != nullptr);
    dn.streaming = plan.routed_streams;
    dn.ksplit = w.slot_planes = plan.routed_ksplit;
    dn.plane_stride = (size_t)T * k * ly.d;
    w.direct = plan.routed_direct;
    w.fused = plan.routed_fused;
    if (plan.routed_fused) return LEXI_OK;   // run_layer launches down + combine once the shared expert's rows are there
    if (plan.routed_direct) {
        dn.out = direct_y; dn.scatter = w.row_token; dn.out_bf16 = direct_bf16;
    }
    if (launch_down(dn, s) != hipSuccess) return LEXI_ERR_LAUNCH;
    mark(3);
    return LEXI_OK;
}

// One layer, arguments already validated.
// `hidden` != null selects the chained block: the MoE input is `u_in` (the normalised hidden state, written by the
// caller or by the previous block's combine), the block's output is added to `hidden` (y may be `hidden` itself), and
// with `u_out` the combine also writes the next block's normalised input.
lexi_status run_layer(const lexi_layer_t& ly, const void* x, void* y, int32_t y_dtype, int32_t T, int32_t k,
                      void* workspace, hipStream_t s, const lexi_routing_out_t* dbg,
                      const lexi_stage_events_t* events = nullptr, const float* hidden = nullptr,
                      const void* u_in = nullptr, void* u_out = nullptr, bool allow_side_stream = true) {
    auto mark = [&](int i) {
        if (events && events->ev[i]) (void)hipEventRecord((hipEvent_t)events->ev[i], s);
    };
    mark(0);
    Workspace w = carve(ly, T, k, workspace);
    const bool bf = ly.dtype == LEXI_BF16;
    if (hidden != nullptr) {
        x = u_in;
    } else if (dbg && dbg->moe_input) {
        if (hipMemcpyAsync(dbg->moe_input, x, (size_t)T * ly.d * (bf ? 2 : 4), hipMemcpyDeviceToDevice, s) != hipSuccess)
            return LEXI_ERR_LAUNCH;
    }
    // routing results land directly in the caller's arrays when those are given
    if (dbg) {
        if (dbg->topk_idx) w.topk_idx = dbg->topk_idx;
        if (dbg->gates) w.gates = dbg->gates;
        if (dbg->counts) w.counts = dbg->counts;
        if (dbg->offsets) w.offsets = dbg->offsets;
        if (dbg->perm) w.perm = dbg->perm;
        if (dbg->inv_perm) w.inv_perm = dbg->inv_perm;
    }

    auto run_shared = [&](hipStream_t st) -> bool {
        const int dense_tiles = (T + kTileTokens - 1) / kTileTokens;
        const bool stream_shared = T <= kStreamDenseRows;
        FfnArgs sg{};
        sg.streaming = stream_shared;
        sg.is_bf16 = bf; sg.in = x; sg.row_token = nullptr; sg.w0 = ly.ws_gate; sg.w1 = ly.ws_up; sg.K = ly.d;
        sg.features = ly.F_shared; sg.M = T; sg.max_tiles = dense_tiles; sg.tile_tokens = kTileTokens;
        sg.sched = nullptr; sg.sched_count = nullptr; sg.out = w.act_shared;
        if (launch_gateup(sg, st) != hipSuccess) return false;
        FfnArgs sd{};
        sd.streaming = stream_shared;
        sd.is_bf16 = bf; sd.in = w.act_shared; sd.row_token = nullptr; sd.w0 = ly.ws_down; sd.w1 = nullptr;
        sd.K = ly.F_shared; sd.features = ly.d; sd.M = T; sd.max_tiles = dense_tiles; sd.tile_tokens = kTileTokens;
        sd.sched = nullptr; sd.sched_count = nullptr; sd.out = w.y_shared;
        sd.ksplit = w.shared_planes = plan_down(ly, T, k, true, false).shared_ksplit;
        sd.plane_stride = (size_t)T * ly.d;
        return launch_down(sd, st) == hipSuccess;
    };
    SideStream* side = (allow_side_stream && ly.F_shared > 0 && T <= kSideStreamMaxT) ? side_stream() : nullptr;
    // the fork/join events are shared by every call on the device: host threads enqueue their layers one at a time
    std::unique_lock<std::mutex> side_lock(g_side_enqueue_mutex, std::defer_lock);
    if (side) {
        side_lock.lock();
        if (hipEventRecord(side->fork, s) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
            return LEXI_ERR_LAUNCH;
        if (!run_shared(side->stream)) return LEXI_ERR_LAUNCH;
        if (hipEventRecord(side->join, side->stream) != hipSuccess) return LEXI_ERR_LAUNCH;
    }

    // Nothing but y to produce (no residual, no normalised copy): the routed down launch may write y itself -- with
    // one active expert and no shared one on the tile schedule, or for a handful of tokens with the combine fused in
    // (plan_down decides).
    const bool direct = hidden == nullptr && u_out == nullptr;
    {
        const lexi_status st = run_routed(ly, x, T, k, w, s, events, true, direct ? y : nullptr, y_dtype == LEXI_BF16);
        if (st != LEXI_OK) return st;
    }
    const bool fused = w.fused;
    if (fused) {
        // the fused launch consumes the shared expert's rows, so the join (or the in-line shared expert) comes first;
        // the stage events keep their meaning: 4 = shared expert done, 3 = routed down done (= 5, combine done)
        if (ly.F_shared > 0) {
            if (side) {
                if (hipStreamWaitEvent(s, side->join, 0) != hipSuccess) return LEXI_ERR_LAUNCH;
            } else if (!run_shared(s)) {
                return LEXI_ERR_LAUNCH;
            }
            mark(4);
        }
        DownCombineArgs f{};
        f.act = w.act; f.w_down = ly.w_down; f.F = ly.F; f.d = ly.d; f.T = T; f.k = k; f.sched = w.sched;
        f.sched_count = w.sched_count; f.inv_perm = w.inv_perm; f.gates = w.gates;
        f.y_shared = ly.F_shared > 0 ? w.y_shared : nullptr; f.y = y; f.y_bf16 = y_dtype == LEXI_BF16;
        if (launch_down_combine(f, s) != hipSuccess) return LEXI_ERR_LAUNCH;
        mark(3);
        if (ly.F_shared == 0) mark(4);
        mark(5);
        return LEXI_OK;
    }

    if (ly.F_shared > 0) {
        if (side) {
            if (hipStreamWaitEvent(s, side->join, 0) != hipSuccess) return LEXI_ERR_LAUNCH;
        } else if (!run_shared(s)) {
            return LEXI_ERR_LAUNCH;
        }
    }
    mark(4);
    if (w.direct) {   // y is complete
        mark(5);
        return LEXI_OK;
    }

    CombineArgs c{};
    c.y_slot = w.y_slot; c.inv_perm = w.inv_perm; c.gates = w.gates;
    c.slot_planes = w.slot_planes; c.slot_plane_stride = (size_t)T * k * ly.d;
    c.shared_planes = w.shared_planes; c.shared_plane_stride = (size_t)T * ly.d;
    c.y_shared = ly.F_shared > 0 ? w.y_shared : nullptr;
    c.x = x; c.x_bf16 = bf;
    c.w_shared_gate = ly.shared_kind == LEXI_SHARED_SIGMOID ? ly.w_shared_gate : nullptr;
    c.residual = hidden; c.u_next = u_out;
    c.T = T; c.d = ly.d; c.k = k; c.y = y; c.y_bf16 = y_dtype == LEXI_BF16;
    if (launch_combine(c, s) != hipSuccess) return LEXI_ERR_LAUNCH;
    mark(5);
    return LEXI_OK;
}

}  // namespace

extern "C" {

lexi_status lexi_pack_weights(const void* src, void* dst, int64_t n_matrices, int32_t rows, int32_t K, int32_t dtype,
                              void* hip_stream) {
    if (dtype != LEXI_F32 && dtype != LEXI_BF16) return LEXI_ERR_DTYPE;
    if (n_matrices < 0 || rows < 16 || rows % 16 != 0 || K < 32 || K % 32 != 0) return LEXI_ERR_SHAPE;
    if (n_matrices == 0) return LEXI_OK;
    if (!src || !dst) return LEXI_ERR_NULL;
    if (misaligned(src) || misaligned(dst) || (dtype == LEXI_F32 && (((uintptr_t)src | (uintptr_t)dst) & 31u)))
        return LEXI_ERR_ALIGN;
    const size_t bytes = (size_t)n_matrices * rows * K * (dtype == LEXI_BF16 ? 2 : 4);
    const char *a = (const char*)src, *b = (const char*)dst;
    if (a < b + bytes && b < a + bytes) return LEXI_ERR_SHAPE;  // overlapping buffers
    if (launch_pack(src, dst, n_matrices, rows, K, dtype == LEXI_BF16, (hipStream_t)hip_stream) != hipSuccess)
        return LEXI_ERR_LAUNCH;
    return LEXI_OK;
}

size_t lexi_moe_workspace_bytes(const lexi_layer_t* layers, int32_t L, int32_t T_max, int32_t k_max) {
    if (!layers || L < 1 || T_max < 0 || k_max < 1) return 0;
    size_t need = 256;
    for (int l = 0; l < L; ++l) {
        if (check_layer(&layers[l]) != LEXI_OK) return 0;
        // a layer cannot be asked for more active experts than it has
        const size_t b = carve(layers[l], T_max, k_max < layers[l].E ? k_max : layers[l].E, nullptr).bytes;
        need = b > need ? b : need;
    }
    return need;
}

lexi_status lexi_moe_layer_forward(const lexi_layer_t* layer, const void* x, void* y, int32_t y_dtype, int32_t T,
                                   int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream,
                                   const lexi_routing_out_t* dbg) {
    lexi_status st = check_call(layer, x, y, y_dtype, T, k, workspace, workspace_bytes, dbg);
    if (st != LEXI_OK || T == 0) return st;
    return run_layer(*layer, x, y, y_dtype, T, k, workspace, (hipStream_t)hip_stream, dbg);
}

lexi_status lexi_moe_layer_forward_static(const lexi_layer_t* layer, const void* x, void* y, int32_t y_dtype, int32_t T,
                                          int32_t k, void* hip_stream, const lexi_routing_out_t* dbg) {
    // validate against the static array's size first: a fake non-null, aligned workspace address stands in until the
    // real one is looked up (check_call only compares it with null and tests its alignment)
    lexi_status st = check_call(layer, x, y, y_dtype, T, k, (const void*)(uintptr_t)256, kStaticScratchBytes, dbg);
    if (st != LEXI_OK || T == 0) return st;
    void* ws = static_scratch();
    if (ws == nullptr) return LEXI_ERR_LAUNCH;
    // every kernel writes the part of the scratch it reads later in the same call, so nothing needs clearing; the
    // shared expert stays on the caller's stream (no library-owned stream or event is created or used)
    return run_layer(*layer, x, y, y_dtype, T, k, ws, (hipStream_t)hip_stream, dbg, nullptr, nullptr, nullptr, nullptr,
                     /*allow_side_stream=*/false);
}

lexi_status lexi_moe_stack_forward_profiled(const lexi_layer_t* layers, int32_t L, const int32_t* k_vec,
                                            const void* x, int64_t x_layer_stride, void* y, int64_t y_layer_stride,
                                            int32_t y_dtype, int32_t T, int32_t mode, void* workspace,
                                            size_t workspace_bytes, void* hip_stream,
                                            const lexi_routing_out_t* dbg_per_layer,
                                            const lexi_stage_events_t* events_per_layer) {
    if (!layers || !k_vec) return LEXI_ERR_NULL;
    if (L < 1 || x_layer_stride < 0 || y_layer_stride < 0) return LEXI_ERR_SHAPE;
    if (mode != LEXI_STACK_INDEPENDENT && mode != LEXI_STACK_CHAINED) return LEXI_ERR_DTYPE;
    const bool chained = mode == LEXI_STACK_CHAINED;
    if (chained && (y_dtype != LEXI_F32 || x_layer_stride != 0)) return LEXI_ERR_DTYPE;   // fp32 hidden state, one input
    // validate every layer before the first launch: an error must leave nothing enqueued
    for (int l = 0; l < L; ++l) {
        const size_t xes = layers[l].dtype == LEXI_BF16 ? 2 : 4;
        const size_t yes = y_dtype == LEXI_BF16 ? 2 : 4;
        const void* xl = x ? (const char*)x + (size_t)l * x_layer_stride * xes : nullptr;
        const void* yl = y ? (const char*)y + (size_t)l * y_layer_stride * yes : nullptr;
        lexi_status st = check_call(&layers[l], xl, yl, y_dtype, T, k_vec[l], workspace, workspace_bytes,
                                    dbg_per_layer ? &dbg_per_layer[l] : nullptr);
        if (st != LEXI_OK) return st;
        if (chained) {
            // one hidden state flows through all blocks: same width and dtype everywhere; outputs either all in one
            // buffer (stride 0: only the last survives) or one full buffer per layer
            if (layers[l].d != layers[0].d || layers[l].dtype != layers[0].dtype) return LEXI_ERR_SHAPE;
            if (y_layer_stride != 0 && y_layer_stride < (int64_t)T * layers[l].d) return LEXI_ERR_SHAPE;
        } else if (L > 1 && T > 0 && y_layer_stride < (int64_t)T * layers[l].d) {
            return LEXI_ERR_SHAPE;  // outputs would overlap
        }
    }
    if (T == 0) return LEXI_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    if (chained) {
        // h_0 = x, widened into the first output buffer; block l reads h_l where block l-1 left it and writes h_{l+1}.
        // The normalised input of block 0 comes from its own kernel, that of every later block from the combine of
        // the block before it; it lives at the start of the workspace unless the caller asked to see it.
        const bool bf = layers[0].dtype == LEXI_BF16;
        auto u_of = [&](int l) -> void* {
            return (dbg_per_layer && dbg_per_layer[l].moe_input) ? dbg_per_layer[l].moe_input : workspace;
        };
        float* h = (float*)y;
        if (launch_widen(x, bf, (size_t)T * layers[0].d, h, s) != hipSuccess) return LEXI_ERR_LAUNCH;
        if (launch_rmsnorm(h, T, layers[0].d, kRmsEps, u_of(0), bf, s) != hipSuccess) return LEXI_ERR_LAUNCH;
        for (int l = 0; l < L; ++l) {
            float* h_out = (float*)y + (size_t)l * y_layer_stride;
            lexi_status st = run_layer(layers[l], nullptr, h_out, LEXI_F32, T, k_vec[l], workspace, s,
                                       dbg_per_layer ? &dbg_per_layer[l] : nullptr,
                                       events_per_layer ? &events_per_layer[l] : nullptr, h, u_of(l),
                                       l + 1 < L ? u_of(l + 1) : nullptr);
            if (st != LEXI_OK) return st;
            h = h_out;
        }
        return LEXI_OK;
    }
    for (int l = 0; l < L; ++l) {
        const size_t xes = layers[l].dtype == LEXI_BF16 ? 2 : 4;
        const size_t yes = y_dtype == LEXI_BF16 ? 2 : 4;
        const void* xl = (const char*)x + (size_t)l * x_layer_stride * xes;
        void* yl = (char*)y + (size_t)l * y_layer_stride * yes;
        lexi_status st = run_layer(layers[l], xl, yl, y_dtype, T, k_vec[l], workspace, s,
                                   dbg_per_layer ? &dbg_per_layer[l] : nullptr,
                                   events_per_layer ? &events_per_layer[l] : nullptr);
        if (st != LEXI_OK) return st;
    }
    return LEXI_OK;
}

lexi_status lexi_moe_stack_forward(const lexi_layer_t* layers, int32_t L, const int32_t* k_vec, const void* x,
                                   int64_t x_layer_stride, void* y, int64_t y_layer_stride, int32_t y_dtype,
                                   int32_t T, int32_t mode, void* workspace, size_t workspace_bytes,
                                   void* hip_stream, const lexi_routing_out_t* dbg_per_layer) {
    return lexi_moe_stack_forward_profiled(layers, L, k_vec, x, x_layer_stride, y, y_layer_stride, y_dtype, T, mode,
                                           workspace, workspace_bytes, hip_stream, dbg_per_layer, nullptr);
}

size_t lexi_moe_profile_workspace_bytes(const lexi_layer_t* layer, int32_t T_max, int32_t k_base, int32_t n_k) {
    if (!layer || check_layer(layer) != LEXI_OK || T_max < 0 || k_base < 1 || k_base > layer->E || n_k < 1 ||
        n_k > kProfileMaxK)
        return 0;
    return carve(*layer, T_max, k_base, nullptr).bytes + align_up((size_t)n_k * T_max * sizeof(float), 256);
}

lexi_status lexi_moe_profile_layer(const lexi_layer_t* layer, const void* x, int32_t T, int32_t k_base,
                                   const int32_t* k_list, int32_t n_k, float* delta, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
    lexi_status st = check_layer(layer);
    if (st != LEXI_OK) return st;
    if (!k_list || !delta) return LEXI_ERR_NULL;
    if (T < 1 || n_k < 1 || n_k > kProfileMaxK) return LEXI_ERR_SHAPE;
    st = check_sizes(layer, T, k_base);
    if (st != LEXI_OK) return st;
    ProfileKList kl{};
    kl.n = n_k;
    for (int i = 0; i < n_k; ++i) {
        if (k_list[i] < 1 || k_list[i] > k_base) return LEXI_ERR_BAD_K;
        kl.k[i] = k_list[i];
    }
    if (!x || !workspace) return LEXI_ERR_NULL;
    if (misaligned(x) || misaligned(workspace) || misaligned(delta)) return LEXI_ERR_ALIGN;
    Workspace w = carve(*layer, T, k_base, workspace);
    if (workspace_bytes < w.bytes + align_up((size_t)n_k * T * sizeof(float), 256)) return LEXI_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    st = run_routed(*layer, x, T, k_base, w, s, nullptr, /*allow_split=*/false);
    if (st != LEXI_OK) return st;
    ProfileArgs p{};
    p.y_slot = w.y_slot; p.inv_perm = w.inv_perm; p.gates = w.gates;
    p.T = T; p.d = layer->d; p.k_base = k_base; p.klist = kl;
    p.part = (float*)((char*)workspace + w.bytes);
    p.delta = delta;
    return launch_profile(p, s) == hipSuccess ? LEXI_OK : LEXI_ERR_LAUNCH;
}

int32_t lexi_moe_down_plan(const lexi_layer_t* layer, int32_t T, int32_t k, int32_t which) {
    if (check_layer(layer) != LEXI_OK || T < 1 || k < 1 || k > layer->E) return -1;
    const DownPlan p = plan_down(*layer, T, k, true, true);
    switch (which) {
        case 0: return p.routed_fused ? 4 : (p.routed_streams ? 0 : (p.routed_direct ? 3 : p.routed_ksplit));
        case 1: return layer->F_shared == 0 ? -1 : (p.shared_streams ? 0 : p.shared_ksplit);
        default: return -1;
    }
}

const char* lexi_strerror(int32_t status) {
    switch (status) {
        case LEXI_OK: return "ok";
        case LEXI_ERR_NULL: return "a required pointer is NULL";
        case LEXI_ERR_SHAPE: return "a dimension violates the shape limits";
        case LEXI_ERR_BAD_K: return "k outside 1..E";
        case LEXI_ERR_DTYPE: return "unknown dtype, shared_kind or mode";
        case LEXI_ERR_WORKSPACE: return "workspace too small";
        case LEXI_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
        case LEXI_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        default: return "unknown status";
    }
}

const char* lexi_moe_version(void) { return "lexi-moe gfx950 0.1"; }

}  // extern "C"
