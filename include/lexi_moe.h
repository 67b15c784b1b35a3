/* lexi_moe.h -- C ABI of the MI355X (gfx950) MoE-layer forward with a per-layer number of active experts.
 *
 * The operation (paper Sec. 2, "Mixture of Experts"):
 *
 *     y = sum_{i in TopK_k(x)} G(x)_i * E_i(x),      G(x) = Softmax(TopK[x * W_g])
 *
 * TopK keeps the k experts with the highest gating scores, Softmax normalises
 * the kept scores, each expert E_i is a SwiGLU FFN
 *     E(x) = Wdown * ( silu(Wgate x) .* (Wup x) ).
 * k is an argument of every call (the UpdateTopk step of Algorithm 1 changes
 * k and nothing else), and a stack of layers takes the static per-layer
 * allocation k* = (k_1 .. k_L) that Algorithm 2 outputs.
 *
 * Conventions that hold for every entry point
 *   - Pointers inside lexi_layer_t, x, y, workspace and every field of
 *     lexi_routing_out_t are DEVICE pointers owned by the caller.  The
 *     lexi_layer_t / lexi_routing_out_t structs themselves, and k_vec, live in
 *     HOST memory.  The library never allocates, frees or keeps a pointer.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL
 *     = the default stream) and the call returns without synchronising.  For
 *     batches of at most 1024 tokens the shared expert's kernels run on a
 *     library-owned side stream that forks from `hip_stream` at the start of
 *     the layer and joins it again before the combine (events, no host
 *     synchronisation): the caller sees plain stream semantics.  That stream
 *     and its two events are created once per device, on first use.
 *   - On error a negative lexi_status is returned and nothing is launched.
 *   - Same inputs give the same output bits on every call; no call leaves
 *     state behind (k=2 then k=8 gives the k=8 result of a fresh call).
 *   - Row-major layouts, last index contiguous:
 *       x, y           [T][d]
 *       w_router       [d][E]   fp32 always (router runs in fp32)
 *       router_bias    [E]      fp32, added to the logits before selection, or NULL
 *       w_gate, w_up   E matrices [F][d]   one row = the input weights of one hidden feature
 *       w_down         E matrices [d][F]   one row = the input weights of one output feature
 *       ws_gate, ws_up one matrix [Fs][d],  ws_down one matrix [d][Fs],  w_shared_gate [d]
 *     Every expert weight MATRIX W[R][K] (all of the above except w_shared_gate) is stored in the PACKED layout
 *     the matrix cores read directly: W is cut into blocks of 16 rows x 32 columns, blocks ordered along K first,
 *     then along R; inside a block the 8-element run (row i, columns 8q..8q+7) sits at run position q*16 + i:
 *         index(r, k) = ((((r/16) * (K/32) + k/32) * 64 + ((k%32)/8) * 16 + r%16) * 8 + k%8
 *     lexi_pack_weights converts row-major matrices into this layout (one-time, per checkpoint load).
 *     dtype LEXI_BF16: x, expert weights and the SwiGLU intermediate are bf16,
 *     accumulation is fp32.  dtype LEXI_F32: everything fp32.
 *   - Shape limits: 1 <= E <= 64, d % 128 == 0, F % 64 == 0, F_shared % 64 == 0,
 *     1 <= k <= E, T >= 0 (T == 0 returns LEXI_OK and launches nothing),
 *     T * k < 2^24; x, the SwiGLU intermediate of the routed experts (T*k rows of F) and of the shared expert
 *     (T rows of F_shared) each stay below 4 GiB.  Every device pointer must be 16-byte aligned.
 *   - Routing semantics: selection on the fp32 logits in the total order (logit
 *     descending, expert index ascending) -- ties go to the lower index, +0 == -0;
 *     inputs must be finite (a token whose logits come out NaN is still routed
 *     safely: a NaN logit ranks below every number, ties to the lower index, and
 *     that token's gates and output row are NaN; no other token is affected).
 *     The k selected experts are kept in rank order ("slots").  Gates are the softmax over the k selected logits (sum to 1).
 *     The fp32 logit is evaluated in a fixed order: d is cut into segments of
 *     128; a segment's partial starts at +0 and takes one fused multiply-add per
 *     element in ascending order; partials are added in ascending order; the
 *     bias is added last.
 *   - Permutation: assignment a = t*k + s (token t, slot s); assignments are
 *     sorted by (expert, token) into contiguous per-expert groups.
 */
#ifndef LEXI_MOE_H
#define LEXI_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LEXI_OK = 0,
    LEXI_ERR_NULL = -1,      /* a required pointer is NULL */
    LEXI_ERR_SHAPE = -2,     /* a dimension violates the shape limits above */
    LEXI_ERR_BAD_K = -3,     /* k < 1 or k > E */
    LEXI_ERR_DTYPE = -4,     /* unknown dtype / shared_kind / mode */
    LEXI_ERR_WORKSPACE = -5, /* workspace_bytes smaller than lexi_moe_workspace_bytes() */
    LEXI_ERR_ALIGN = -6,     /* a device pointer is not 16-byte aligned */
    LEXI_ERR_LAUNCH = -7     /* the HIP runtime refused a launch */
} lexi_status;

typedef enum { LEXI_F32 = 0, LEXI_BF16 = 1 } lexi_dtype;
typedef enum { LEXI_SHARED_NONE = 0, LEXI_SHARED_UNGATED = 1, LEXI_SHARED_SIGMOID = 2 } lexi_shared_kind;

/* One MoE layer (Sec. 2: gate W_g and experts E_i).  Host struct, device pointers. */
typedef struct {
    int32_t d, E, F, F_shared;  /* F_shared = 0: no shared expert (two shared experts = one of twice the width) */
    int32_t dtype;              /* lexi_dtype of x, expert weights and the SwiGLU intermediate */
    int32_t shared_kind;        /* lexi_shared_kind */
    const float* w_router;      /* [d][E] */
    const float* router_bias;   /* [E] or NULL */
    const void* w_gate;         /* E packed matrices [F][d] */
    const void* w_up;           /* E packed matrices [F][d] */
    const void* w_down;         /* E packed matrices [d][F] */
    const void* ws_gate;        /* packed [Fs][d] or NULL */
    const void* ws_up;          /* packed [Fs][d] or NULL */
    const void* ws_down;        /* packed [d][Fs] or NULL */
    const void* w_shared_gate;  /* [d] (LEXI_SHARED_SIGMOID) or NULL */
} lexi_layer_t;

/* Optional routing outputs; any field may be NULL.  Device pointers. */
typedef struct {
    int32_t* topk_idx;  /* [T][k]  selected experts in rank order */
    float* gates;       /* [T][k]  softmax over the selected logits */
    int32_t* counts;    /* [E]     assignments per expert */
    int32_t* offsets;   /* [E+1]   exclusive scan of counts */
    int32_t* perm;      /* [T*k]   position -> assignment t*k+s */
    int32_t* inv_perm;  /* [T*k]   assignment -> position */
    void* moe_input;    /* [T][d]  of the layer dtype: the input the MoE block actually consumed (a copy of x; in the
                           chained mode the normalised hidden state) */
} lexi_routing_out_t;

/* Stack modes. */
typedef enum { LEXI_STACK_INDEPENDENT = 0, LEXI_STACK_CHAINED = 1 } lexi_stack_mode;

/* Re-layout of expert weights (the E_i of Sec. 2) from row-major into the packed layout described above.
 *   src: device, n_matrices row-major matrices [rows][K] back to back; dst: device, same size, must not overlap src;
 *   rows % 16 == 0, K % 32 == 0, dtype = lexi_dtype of the elements.  Asynchronous on hip_stream. */
lexi_status lexi_pack_weights(const void* src, void* dst, int64_t n_matrices, int32_t rows, int32_t K, int32_t dtype,
                              void* hip_stream);

/* Bytes of device workspace that any call with these layers, T <= T_max and k <= k_max needs (per layer k is
 * at most the layer's E, so k_max may exceed the E of some layers of a stack).
 * layers: host array[L].  Returns 0 if an argument is invalid. */
size_t lexi_moe_workspace_bytes(const lexi_layer_t* layers, int32_t L, int32_t T_max, int32_t k_max);

/* f_moe(X; k) for one layer (Sec. 2; Algorithm 1's UpdateTopk + f_moe).
 *   x [T][d] of layer->dtype; y [T][d] of y_dtype (LEXI_F32, or LEXI_BF16 = nearest-even rounding of the fp32 result);
 *   workspace: device scratch of at least lexi_moe_workspace_bytes(layer, 1, T, k) bytes, contents undefined on
 *   entry and exit; dbg: NULL or where to copy the routing decision. */
lexi_status lexi_moe_layer_forward(const lexi_layer_t* layer, const void* x, void* y, int32_t y_dtype, int32_t T,
                                   int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream,
                                   const lexi_routing_out_t* dbg);

/* lexi_moe_layer_forward for callers that cannot allocate device memory or carry a workspace around: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the workspace, same
 * kernels, same result bits.  The scratch lives in a static device array inside the library (64 MiB; each GPU the
 * library runs on holds its copy until the process ends), whose address is looked up on the first call on a device.
 * The call allocates nothing, frees nothing, and creates no stream or event (a shared expert runs on `hip_stream`).
 *   Limit: the call must need at most 64 MiB of workspace (lexi_moe_workspace_bytes(layer, 1, T, k) <= 67108864:
 *   decode-sized batches of every workload shape here), otherwise LEXI_ERR_WORKSPACE and nothing is launched.
 *   All calls on one GPU share the one array: calls that overlap in time on the same GPU (different streams or host
 *   threads) race; calls on one stream are ordered and safe.  The array keeps the last call's contents; no kernel
 *   relies on them. */
lexi_status lexi_moe_layer_forward_static(const lexi_layer_t* layer, const void* x, void* y, int32_t y_dtype, int32_t T,
                                          int32_t k, void* hip_stream, const lexi_routing_out_t* dbg);

/* A stack of L layers with the static per-layer allocation k_vec = (k_1 .. k_L) (Sec. 1; output of Algorithm 2).
 *   layers: host array[L]; k_vec: HOST int32[L].
 *   mode LEXI_STACK_INDEPENDENT: layer l reads x + l*x_layer_stride elements and writes y + l*y_layer_stride elements
 *   (stride 0 for x = every layer reads the same X, as in Algorithm 1's per-layer profiling on one random X).
 *   mode LEXI_STACK_CHAINED: pre-norm residual blocks, the setting of end-to-end inference (Sec. 3) reduced to its
 *   MoE blocks: h_0 = x [T][d] (x_layer_stride must be 0);  u_l = h_l / sqrt(mean_j h_l[j]^2 + 1e-6) rounded to the
 *   layer dtype;  h_{l+1} = h_l + f_moe_l(u_l; k_l), hidden state in fp32 (y_dtype must be LEXI_F32).  y + l*
 *   y_layer_stride receives h_{l+1}; stride 0 keeps only the final hidden state.  All layers share d and dtype.
 *   dbg_per_layer: NULL or host array[L]. */
lexi_status lexi_moe_stack_forward(const lexi_layer_t* layers, int32_t L, const int32_t* k_vec, const void* x,
                                   int64_t x_layer_stride, void* y, int64_t y_layer_stride, int32_t y_dtype,
                                   int32_t T, int32_t mode, void* workspace, size_t workspace_bytes,
                                   void* hip_stream, const lexi_routing_out_t* dbg_per_layer);

/* Stage boundaries of one layer, for timing from outside with HIP events: the library records ev[i] on the
 * stream at boundary i.  0 = layer start, 1 = routing done (router, top-k, gates, permutation), 2 = routed gate/up
 * GEMM + SwiGLU done, 3 = routed down GEMM done, 4 = shared expert done, 5 = combine done.  A NULL event is
 * skipped.  Events are hipEvent_t handles owned by the caller (host struct).  A call for a handful of tokens whose
 * down projection and combine are one launch (it consumes the shared expert's rows) records 4 BEFORE that launch and
 * 3 and 5 after it. */
#define LEXI_N_STAGE_EVENTS 6
typedef struct {
    void* ev[LEXI_N_STAGE_EVENTS];
} lexi_stage_events_t;

/* lexi_moe_stack_forward plus stage events: events_per_layer is a host array[L] (or NULL = no events).
 * Same kernels, same launch order, same results; the only extra work is the event records. */
lexi_status lexi_moe_stack_forward_profiled(const lexi_layer_t* layers, int32_t L, const int32_t* k_vec,
                                            const void* x, int64_t x_layer_stride, void* y, int64_t y_layer_stride,
                                            int32_t y_dtype, int32_t T, int32_t mode, void* workspace,
                                            size_t workspace_bytes, void* hip_stream,
                                            const lexi_routing_out_t* dbg_per_layer,
                                            const lexi_stage_events_t* events_per_layer);

/* One iteration of the Stage-1 top-k perturbation profiling (Algorithm 1) on one input X:
 *     delta[i] = || f_moe(X; k_list[i]) - f_moe(X; k_base) ||_F ,   1 <= k_list[i] <= k_base <= E,  n_k <= 64.
 *   The selection order is total, so TopK_k is a prefix of TopK_{k_base}: one routing pass and one pass of the expert
 *   GEMMs at k_base serve every k of the list (the algorithm as printed runs 1 + n_k full passes), and a shared
 *   expert, which adds the same vector to both outputs, drops out of the difference.
 *   x [T][d] of layer->dtype (T >= 1); k_list: HOST int32[n_k]; delta: DEVICE float[n_k], receives this X's
 *   deviations (averaging over iterations, the algorithm's last step, is the caller's).  workspace: device scratch of
 *   at least lexi_moe_profile_workspace_bytes(layer, T, k_base, n_k) bytes.  Asynchronous on hip_stream. */
size_t lexi_moe_profile_workspace_bytes(const lexi_layer_t* layer, int32_t T_max, int32_t k_base, int32_t n_k);
lexi_status lexi_moe_profile_layer(const lexi_layer_t* layer, const void* x, int32_t T, int32_t k_base,
                                   const int32_t* k_list, int32_t n_k, float* delta, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);

/* LExI Stage 2 (Algorithm 2): evolutionary search for the per-layer allocation k* = (k_1 .. k_L) that minimises
 * phi(k) = sum_j D[j][k_j] subject to sum_j k_j = B and k_min <= k_j <= k_max.  HOST function, HOST pointers, no GPU.
 *   D: [L][k_max + 1] doubles, entry [j][k] = Stage-1 loss of layer j at top-k = k (entries below k_min are not read);
 *   n_pop >= 2 individuals, g_max generations, eta_mut = per-layer probability of a balanced +-1 move, seed of the
 *   counter-based random stream (same arguments, same result, on any machine);
 *   k_out: int32[L] receives k*; phi_out: NULL or receives phi(k*).
 *   The reading of the steps the paper leaves open (tournaments of two, uniform crossover, balanced mutation, greedy
 *   projection, elitist truncation to n_pop) is written out at the top of csrc/stage2.hip.
 *   Returns LEXI_ERR_BAD_K when no feasible vector exists (B outside L*k_min .. L*k_max). */
lexi_status lexi_allocate_topk(const double* D, int32_t L, int32_t B, int32_t k_min, int32_t k_max, int32_t n_pop,
                               int32_t g_max, double eta_mut, uint64_t seed, int32_t* k_out, double* phi_out);

/* Static description of a status code. */
const char* lexi_strerror(int32_t status);

/* Names of the device kernels one call launches are stable; this returns the library's version string. */
const char* lexi_moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LEXI_MOE_H */
