/* CPU oracle for the MoE layer forward with a per-layer number of active experts.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests and the benchmark's CPU-baseline leg have a plain,
 * slow, independent statement of what the layer computes.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * What it computes (paper Sec. 2, "Mixture of Experts"):
 *     y = sum_{i in TopK_k} G(x)_i * E_i(x),   G(x) = Softmax(TopK[x * W_g])
 * with k settable per call (the UpdateTopk step of Algorithm 1) and, for a
 * stack, a static per-layer vector k* = (k_1 .. k_L) (output of Algorithm 2).
 * Each E_i is a SwiGLU FFN:  E(x) = Wdown * ( silu(Wgate x) .* (Wup x) ).
 *
 * Readings of points the paper leaves open (every one is also listed in the
 * design document):
 *   - selection runs on the raw fp32 logits; the total order is (logit
 *     descending, expert index ascending), so ties go to the lower index and
 *     +0.0 == -0.0; the k selected experts are kept in that rank order;
 *   - the softmax runs over the k selected logits only (equivalently: full
 *     softmax, then renormalise over the selected), so gates sum to 1;
 *   - the fp32 logit of (token, expert) is evaluated in ONE fixed order so
 *     that another implementation can reproduce its bits: the hidden
 *     dimension is cut into consecutive segments of 128; inside a segment the
 *     partial sum starts at +0.0f and is updated by a single-rounding fused
 *     multiply-add per element in ascending order; the segment partials are
 *     then added in ascending order with plain fp32 additions (the first
 *     partial is taken as is), and the optional bias is added last;
 *   - everything after the routing decision is evaluated in fp64.  For bf16
 *     layers the SwiGLU intermediate may be rounded to bf16 (through fp32) at
 *     the one point where a bf16 implementation stores it ("round_act");
 *   - the permutation is the stable counting sort of the (token, slot) pairs
 *     by expert: inside one expert's group tokens ascend;
 *   - a shared expert is added after the routed sum, scaled by 1 (ungated) or
 *     by sigmoid(x . w_shared_gate); two ungated shared experts are the same
 *     as one whose inner dimension is the concatenation of both.
 *
 * Layouts (row-major): x [T][d]; w_router [d][E] fp32; router_bias [E];
 * w_gate, w_up [E][F][d]; w_down [E][d][F]; ws_gate, ws_up [Fs][d];
 * ws_down [d][Fs]; w_shared_gate [d].  dtype 0 = fp32, 1 = bf16 stored as
 * uint16 bit patterns (widened exactly).  All pointers are host pointers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t d, E, F, F_shared;
    int32_t dtype;       /* 0 = fp32, 1 = bf16 */
    int32_t shared_kind; /* 0 none, 1 ungated, 2 sigmoid-gated */
    const float* w_router;
    const float* router_bias; /* may be NULL */
    const void* w_gate;
    const void* w_up;
    const void* w_down;
    const void* ws_gate;
    const void* ws_up;
    const void* ws_down;
    const void* w_shared_gate;
} oracle_layer;

#define ROUTER_SEGMENT 128

static inline float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static inline float f32_round_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return f;
}

/* element i of a tensor of the layer's dtype, widened exactly to fp32 */
static inline float load_elem(const void* p, int dtype, size_t i) {
    return dtype == 0 ? ((const float*)p)[i] : bf16_to_f32(((const uint16_t*)p)[i]);
}

int lexi_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Router logits in the fixed fp32 order (Sec. 2: x * W_g).  logits [T][E]. */
int lexi_oracle_router_logits(const oracle_layer* ly, const void* x, int32_t T, float* logits) {
    const int d = ly->d, E = ly->E;
    if (d % ROUTER_SEGMENT != 0) return -2;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            float total = 0.0f;
            for (int seg = 0; seg < d / ROUTER_SEGMENT; ++seg) {
                float p = 0.0f;
                for (int j = seg * ROUTER_SEGMENT; j < (seg + 1) * ROUTER_SEGMENT; ++j) {
                    float xv = load_elem(x, ly->dtype, (size_t)t * d + j);
                    p = fmaf(xv, ly->w_router[(size_t)j * E + e], p);
                }
                total = (seg == 0) ? p : total + p;
            }
            if (ly->router_bias) total = total + ly->router_bias[e];
            logits[(size_t)t * E + e] = total;
        }
    }
    return 0;
}

/* TopK[.]: the k experts first in the order (logit descending, index ascending).  topk_idx [T][k]. */
int lexi_oracle_topk(const float* logits, int32_t T, int32_t E, int32_t k, int32_t* topk_idx) {
    if (k < 1 || k > E) return -3;
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (size_t)t * E;
        char* taken = (char*)calloc((size_t)E, 1);
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e; /* strict '>' : an equal logit never displaces a lower index */
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + s] = best;
        }
        free(taken);
    }
    return 0;
}

/* Softmax over the selected logits (Sec. 2: G = Softmax(TopK[.])), fp64, stored fp32.  gates [T][k]. */
int lexi_oracle_gates(const float* logits, const int32_t* topk_idx, int32_t T, int32_t E, int32_t k, float* gates) {
    for (int t = 0; t < T; ++t) {
        const float* l = logits + (size_t)t * E;
        const int32_t* sel = topk_idx + (size_t)t * k;
        double lmax = (double)l[sel[0]]; /* slot 0 holds the largest selected logit */
        double denom = 0.0;
        for (int s = 0; s < k; ++s) denom += exp((double)l[sel[s]] - lmax);
        for (int s = 0; s < k; ++s) gates[(size_t)t * k + s] = (float)(exp((double)l[sel[s]] - lmax) / denom);
    }
    return 0;
}

/* Token-to-expert permutation: assignments a = t*k+s sorted by (expert, token).
 * counts [E], offsets [E+1], perm [T*k] (position -> assignment), inv_perm [T*k] (assignment -> position). */
int lexi_oracle_permutation(const int32_t* topk_idx, int32_t T, int32_t E, int32_t k, int32_t* counts,
                            int32_t* offsets, int32_t* perm, int32_t* inv_perm) {
    int32_t pos = 0;
    for (int e = 0; e < E; ++e) {
        offsets[e] = pos;
        for (int t = 0; t < T; ++t)
            for (int s = 0; s < k; ++s)
                if (topk_idx[(size_t)t * k + s] == e) {
                    perm[pos] = t * k + s;
                    inv_perm[t * k + s] = pos;
                    ++pos;
                }
        counts[e] = pos - offsets[e];
    }
    offsets[E] = pos;
    return pos == T * k ? 0 : -4;
}

/* One SwiGLU FFN on one token row: y[j] = sum_f a[f] * Wd[j][f], a[f] = silu(Wg[f].x) * (Wu[f].x).
 * wg, wu: [F][d]; wd: [d][F]; fp64 accumulation in ascending index order.  y [d] fp64. */
static void ffn_row(const void* xrow, const void* wg, const void* wu, const void* wd, int dtype, int d, int F,
                    int round_act, double* a, double* y) {
    for (int f = 0; f < F; ++f) {
        double hg = 0.0, hu = 0.0;
        for (int j = 0; j < d; ++j) {
            double xv = (double)load_elem(xrow, dtype, (size_t)j);
            hg += xv * (double)load_elem(wg, dtype, (size_t)f * d + j);
            hu += xv * (double)load_elem(wu, dtype, (size_t)f * d + j);
        }
        double act = hg / (1.0 + exp(-hg)) * hu;
        if (round_act && dtype == 1) act = (double)f32_round_bf16((float)act);
        a[f] = act;
    }
    for (int j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int f = 0; f < F; ++f) acc += a[f] * (double)load_elem(wd, dtype, (size_t)j * F + f);
        y[j] = acc;
    }
}

/* Output of routed expert e (0 <= e < E) or of the shared expert (e == -1, unscaled) for token row t of x. */
int lexi_oracle_expert_ffn(const oracle_layer* ly, int32_t e, const void* x, int32_t t, int32_t round_act, double* y) {
    const int d = ly->d;
    const size_t es = ly->dtype == 0 ? 4 : 2;
    const char* xrow = (const char*)x + (size_t)t * d * es;
    if (e >= 0) {
        if (e >= ly->E) return -2;
        const int F = ly->F;
        double* a = (double*)malloc(sizeof(double) * (size_t)F);
        const size_t off = (size_t)e * F * d * es;
        ffn_row(xrow, (const char*)ly->w_gate + off, (const char*)ly->w_up + off, (const char*)ly->w_down + off,
                ly->dtype, d, F, round_act, a, y);
        free(a);
    } else {
        if (ly->F_shared <= 0) return -2;
        const int F = ly->F_shared;
        double* a = (double*)malloc(sizeof(double) * (size_t)F);
        ffn_row(xrow, ly->ws_gate, ly->ws_up, ly->ws_down, ly->dtype, d, F, round_act, a, y);
        free(a);
    }
    return 0;
}

/* Coefficient of the shared expert for token t: 1 (ungated) or sigmoid(x_t . w_shared_gate). */
double lexi_oracle_shared_coeff(const oracle_layer* ly, const void* x, int32_t t) {
    if (ly->shared_kind != 2) return 1.0;
    double z = 0.0;
    for (int j = 0; j < ly->d; ++j)
        z += (double)load_elem(x, ly->dtype, (size_t)t * ly->d + j) * (double)load_elem(ly->w_shared_gate, ly->dtype, (size_t)j);
    return 1.0 / (1.0 + exp(-z));
}

/* Whole layer: routing for all T tokens, expert FFNs + gate-weighted sum (+ shared expert) for the tokens in
 * token_list (n_tokens entries; NULL = all T tokens, then n_tokens must equal T).
 *   out      [n_tokens][d] fp64
 * Optional routing outputs (any may be NULL): logits [T][E], topk_idx [T][k], gates [T][k], counts [E],
 * offsets [E+1], perm [T*k], inv_perm [T*k].
 * routing_only != 0 skips the FFN part (out may then be NULL). */
int lexi_oracle_moe_layer(const oracle_layer* ly, const void* x, int32_t T, int32_t k, const int32_t* token_list,
                          int32_t n_tokens, int32_t round_act, int32_t routing_only, double* out, float* logits_out,
                          int32_t* topk_idx_out, float* gates_out, int32_t* counts_out, int32_t* offsets_out,
                          int32_t* perm_out, int32_t* inv_perm_out) {
    const int d = ly->d, E = ly->E;
    if (k < 1 || k > E) return -3;
    if (T < 0 || (token_list == NULL && n_tokens != T)) return -2;
    if (T == 0) return 0;
    float* logits = (float*)malloc(sizeof(float) * (size_t)T * E);
    int32_t* sel = (int32_t*)malloc(sizeof(int32_t) * (size_t)T * k);
    float* gates = (float*)malloc(sizeof(float) * (size_t)T * k);
    int32_t* counts = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
    int32_t* offsets = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)T * k);
    int32_t* inv_perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)T * k);
    int rc = lexi_oracle_router_logits(ly, x, T, logits);
    if (rc == 0) rc = lexi_oracle_topk(logits, T, E, k, sel);
    if (rc == 0) rc = lexi_oracle_gates(logits, sel, T, E, k, gates);
    if (rc == 0) rc = lexi_oracle_permutation(sel, T, E, k, counts, offsets, perm, inv_perm);
    if (rc == 0 && !routing_only) {
#pragma omp parallel
        {
            double* y = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
            for (int n = 0; n < n_tokens; ++n) {
                const int t = token_list ? token_list[n] : n;
                double* o = out + (size_t)n * d;
                for (int j = 0; j < d; ++j) o[j] = 0.0;
                for (int s = 0; s < k; ++s) { /* slot order = rank order */
                    lexi_oracle_expert_ffn(ly, sel[(size_t)t * k + s], x, t, round_act, y);
                    const double gte = (double)gates[(size_t)t * k + s];
                    for (int j = 0; j < d; ++j) o[j] += gte * y[j];
                }
                if (ly->shared_kind != 0 && ly->F_shared > 0) {
                    lexi_oracle_expert_ffn(ly, -1, x, t, round_act, y);
                    const double c = lexi_oracle_shared_coeff(ly, x, t);
                    for (int j = 0; j < d; ++j) o[j] += c * y[j];
                }
            }
            free(y);
        }
    }
    if (rc == 0) {
        if (logits_out) memcpy(logits_out, logits, sizeof(float) * (size_t)T * E);
        if (topk_idx_out) memcpy(topk_idx_out, sel, sizeof(int32_t) * (size_t)T * k);
        if (gates_out) memcpy(gates_out, gates, sizeof(float) * (size_t)T * k);
        if (counts_out) memcpy(counts_out, counts, sizeof(int32_t) * (size_t)E);
        if (offsets_out) memcpy(offsets_out, offsets, sizeof(int32_t) * (size_t)(E + 1));
        if (perm_out) memcpy(perm_out, perm, sizeof(int32_t) * (size_t)T * k);
        if (inv_perm_out) memcpy(inv_perm_out, inv_perm, sizeof(int32_t) * (size_t)T * k);
    }
    free(logits); free(sel); free(gates); free(counts); free(offsets); free(perm); free(inv_perm);
    return rc;
}
