/*
 * CPU oracle for the capacity-aware MoE layer forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition the GPU
 * library is checked against.  Only the tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it; the product path never does.  It shares no code
 * with the HIP kernels.
 *
 * Every function follows a passage of "Capacity-Aware Inference: Mitigating the
 * Straggler Effect in Mixture of Experts" (arXiv 2503.05066), cited at the function.
 * Loops are written in the order of the definitions: no blocking, no fusion.
 *
 * Conventions the paper leaves open (each is a reading of this build, not a fact
 * of the paper; "parity unpinned" applies to exactly these):
 *   - the fp32 operation sequence of the softmax (orc_softmax_scores),
 *   - ties in the top-k go to the lower expert id, ties at the capacity threshold
 *     to the lower token index, and exactly `cap` candidates are kept,
 *   - rows of the dispatch plan are expert-major, ascending token inside an expert,
 *   - token t lives on simulated device t / (N/G), which hosts experts
 *     [b*E/G, (b+1)*E/G),
 *   - the generator behind the Random metric (orc_pair_hash) and the encoding of the
 *     multimodal strategies as a class per token.
 *
 * All matrices are row-major host arrays.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_MODE_NONE = 0, ORC_MODE_TOKEN_DROP = 1, ORC_MODE_EXPANDED_DROP = 2 };
enum { ORC_SCOPE_LOCAL = 0, ORC_SCOPE_GLOBAL = 1, ORC_SCOPE_LOCAL_DEVICE = 2, ORC_SCOPE_GLOBAL_DEVICE = 3 };

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of host threads the parallel loops use from now on (timing only; results do not depend on it). */
void orc_set_num_threads(int n) {
    if (n >= 1) omp_set_num_threads(n);
}

/* ---------------------------------------------------------------------------
 * Router logits: the gate projection G(x) inside Eq. (1), `self.gate(x)` in Alg. 1 / Alg. 2.
 * logits[t,e] = sum_j x[t,j] * w[e,j] (+ bias[e]); summed in fp64, stored as fp32.
 * ------------------------------------------------------------------------- */
void orc_router_logits(const float* x, const float* w, const float* bias, int N, int d, int E,
                       float* logits) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < N; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) acc += (double)x[(size_t)t * d + j] * (double)w[(size_t)e * d + j];
            if (bias) acc += (double)bias[e];
            logits[(size_t)t * E + e] = (float)acc;
        }
    }
}

/* ---------------------------------------------------------------------------
 * Softmax over experts, Eq. (1); the softmax of Alg. 1 / Alg. 2.
 *
 * The scores rank tokens, i.e. they decide integers, so they are computed in the
 * precision the GPU computes them in (fp32) by a fixed operation sequence:
 *   m = max_e l[e];  z = l[e] - m
 *   p = 0                       if z < -80
 *   p = 2^n * poly(r) otherwise, n = rint(z*log2(e)), r = z - n*ln2 (two fused steps),
 *       poly = degree-7 Taylor polynomial of exp evaluated by Horner with fused
 *       multiply-adds,
 *   S = p[0] + p[1] + ... in ascending expert order,  s[e] = p[e] / S.
 * The cut at -80 keeps p and p/S normal numbers for any E up to 1024.
 * Compile with -ffp-contract=off: every rounding below is explicit.
 * ------------------------------------------------------------------------- */
static float orc_exp_nonpositive(float z) {
    if (z < -80.0f) return 0.0f;
    const float n = rintf(z * 0x1.715476p+0f);
    float r = fmaf(n, -0x1.62e400p-1f, z);
    r = fmaf(n, -0x1.7f7d1cp-20f, r);
    float q = 0x1.a01a02p-13f;          /* 1/5040 */
    q = fmaf(q, r, 0x1.6c16c2p-10f);    /* 1/720  */
    q = fmaf(q, r, 0x1.111112p-7f);     /* 1/120  */
    q = fmaf(q, r, 0x1.555556p-5f);     /* 1/24   */
    q = fmaf(q, r, 0x1.555556p-3f);     /* 1/6    */
    q = fmaf(q, r, 0.5f);
    q = fmaf(q, r, 1.0f);
    q = fmaf(q, r, 1.0f);
    return ldexpf(q, (int)n);
}

void orc_softmax_scores(const float* logits, int N, int E, float* scores) {
    for (int t = 0; t < N; ++t) {
        const float* l = logits + (size_t)t * E;
        float* s = scores + (size_t)t * E;
        float m = l[0];
        for (int e = 1; e < E; ++e)
            if (l[e] > m) m = l[e];
        float sum = 0.0f;
        for (int e = 0; e < E; ++e) {
            s[e] = orc_exp_nonpositive(l[e] - m);
            sum = sum + s[e];
        }
        for (int e = 0; e < E; ++e) s[e] = s[e] / sum;
    }
}

/* ---------------------------------------------------------------------------
 * Top-k of the post-softmax scores, Eq. (1); `scores.topk(k, dim=1)` in Alg. 1.
 * Selection by repeated maximum; equal scores go to the lower expert id.
 * Output slot j holds the (j+1)-th best expert of the token.
 * ------------------------------------------------------------------------- */
void orc_topk(const float* scores, int N, int E, int k, int32_t* topk_idx, float* topk_score) {
    uint8_t* taken = (uint8_t*)malloc((size_t)E);
    for (int t = 0; t < N; ++t) {
        const float* s = scores + (size_t)t * E;
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || s[e] > s[best]) best = e;
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + j] = best;
            topk_score[(size_t)t * k + j] = s[best];
        }
    }
    free(taken);
}

/* ---------------------------------------------------------------------------
 * Expert capacity C = gamma * N_bar, N_bar = N*k/E (Sec. 3.1 and Sec. 4); as an
 * integer it is evaluated as in Alg. 1: gamma times (N*k), divided by E, truncated.
 * `seg_tokens` is the number of tokens the constraint ranges over (all N, or the
 * N/G tokens of one device when capacity is enforced locally, Sec. 4).  The result is
 * clamped to seg_tokens: an expert cannot hold more tokens than exist.
 * ------------------------------------------------------------------------- */
int orc_capacity(double gamma, int seg_tokens, int k, int E) {
    if (isinf(gamma) && gamma > 0) return seg_tokens;
    double c = gamma * (double)((long long)seg_tokens * (long long)k) / (double)E;
    if (!(c > 0.0)) return 0;
    if (c >= (double)seg_tokens) return seg_tokens;
    return (int)c;
}

/* ---------------------------------------------------------------------------
 * Candidate set of every token.
 *   Token Drop (Alg. 1): the token's top-k experts.  Over-selection (Sec. 5.2 "Effectiveness
 *   of Expanded Drop", over-selection ratio m; appendix table with m = 2k, 3k): the list
 *   handed in is the token's top-(k+m) instead, and `k` below is that list's width, while the
 *   capacity keeps using the model's k.
 *   Expanded Drop (Alg. 2, Sec. 4 "Expanded Drop"): top-k plus all m = E/G experts
 *   hosted on the token's own device.  A set: an expert that is both counts once.
 * cand is a dense [N,E] 0/1 matrix.
 * ------------------------------------------------------------------------- */
void orc_candidates(const int32_t* topk_idx, int N, int E, int k, int G, int mode, uint8_t* cand) {
    const int tokens_per_dev = N / G, experts_per_dev = E / G;
    memset(cand, 0, (size_t)N * E);
    for (int t = 0; t < N; ++t) {
        for (int j = 0; j < k; ++j) cand[(size_t)t * E + topk_idx[(size_t)t * k + j]] = 1;
        if (mode == ORC_MODE_EXPANDED_DROP) {
            const int dev = t / tokens_per_dev;
            for (int e = dev * experts_per_dev; e < (dev + 1) * experts_per_dev; ++e) cand[(size_t)t * E + e] = 1;
        }
    }
}

/* ---------------------------------------------------------------------------
 * Ranked drop, Eqs. (8)-(10) (threshold tau, kept set T_J, mask M_J) and the
 * column-wise topk(cap) of Alg. 1 / Alg. 2.
 *
 * A capacity segment is one expert over the tokens the constraint ranges over:
 * scope GLOBAL - all N tokens; scope LOCAL - the N/G tokens of one device (Sec. 4:
 * constraints are applied to the tokens within each local device).  In every segment
 * the candidates are sorted by importance and the first `cap` are kept.  Mode NONE
 * keeps every candidate.
 *
 * Importance of a candidate (token t, expert e), Sec. 4 "metrics":
 *   SCORE          its gating score s[t,e] (higher is kept first)
 *   ORDER          earlier tokens are kept first (later ones are discarded once the
 *                  capacity is filled)
 *   REVERSE_ORDER  later tokens are kept first
 *   RANDOM         an independent uniform draw per pair: the 29 high bits of a 32-bit
 *                  integer hash of (seed, t*E + e) - a counter-based generator, so that
 *                  any implementation draws the same numbers
 * Multimodal strategies (Sec. "Extension to Multimodal Mixture of Experts": "Image First",
 * "Text First", "Uniform"): an optional
 * class per token (0..3) ranks before the metric - a candidate of a lower class is
 * dropped before any candidate of a higher class.  Image First = image tokens class 0,
 * text tokens class 1; Uniform = no classes.
 * Equal importance goes to the lower token index, then (only relevant when several experts
 * share a budget) to the lower expert id.
 *
 * Granularity (Sec. 5.2, "Advanced Variant: Device-Level Capacity-Aware Inference"): with a
 * *_DEVICE scope the constraint bounds the aggregated load of the E/G experts of one device,
 * N_1 + ... + N_nl <= n_l * gamma * N_bar, instead of each expert: all candidate pairs of
 * the device's experts are ranked together and the best `budget` are kept.  (The paper gives
 * the constraint, not the selection rule; ranking by the same metric is this build's reading.)
 * keep is a dense [N,E] 0/1 matrix.  Returns the number of kept pairs.
 * ------------------------------------------------------------------------- */
enum { ORC_METRIC_SCORE = 0, ORC_METRIC_ORDER = 1, ORC_METRIC_REVERSE_ORDER = 2, ORC_METRIC_RANDOM = 3 };

/* 32-bit integer hash (two multiply-xorshift rounds); the counter is offset by the seed */
uint32_t orc_pair_hash(uint32_t seed, uint32_t counter) {
    uint32_t x = counter + seed * 0x9E3779B9u;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

typedef struct { int cls; double value; int32_t expert; int32_t token; } orc_cand_t;

static int orc_cand_cmp(const void* a, const void* b) {
    const orc_cand_t* p = (const orc_cand_t*)a;
    const orc_cand_t* q = (const orc_cand_t*)b;
    if (p->cls != q->cls) return p->cls > q->cls ? -1 : 1;
    if (p->value > q->value) return -1;
    if (p->value < q->value) return 1;
    if (p->token != q->token) return p->token < q->token ? -1 : 1;
    return (p->expert > q->expert) - (p->expert < q->expert);
}

static double orc_importance(const float* scores, int E, int t, int e, int metric, uint32_t seed) {
    switch (metric) {
        case ORC_METRIC_ORDER: return -(double)t;
        case ORC_METRIC_REVERSE_ORDER: return (double)t;
        case ORC_METRIC_RANDOM: return (double)(orc_pair_hash(seed, (uint32_t)t * (uint32_t)E + (uint32_t)e) >> 3);
        default: return (double)scores[(size_t)t * E + e];
    }
}

/* Device-level budget (Sec. 5.2 "Device-Level Capacity-Aware Inference"): the experts of one
 * device together hold at most n_l * gamma * N_bar pairs, n_l = E/G; as an integer it is
 * evaluated like the expert capacity: gamma times (N*k*n_l), divided by E, truncated. */
int orc_device_budget(double gamma, int seg_tokens, int k, int E, int experts_per_device) {
    if (isinf(gamma) && gamma > 0) return seg_tokens * experts_per_device; /* no limit: every possible pair */
    double c = gamma * (double)((long long)seg_tokens * k * experts_per_device) / (double)E;
    if (!(c > 0.0)) return 0;
    if (c >= (double)seg_tokens * (double)experts_per_device) return seg_tokens * experts_per_device;
    return (int)c;
}

int64_t orc_capacity_drop(const float* scores, const uint8_t* cand, int N, int E, int k, int G, int mode,
                          int scope, double gamma, int metric, const uint8_t* token_class, uint32_t seed,
                          uint8_t* keep) {
    const int per_device = scope == ORC_SCOPE_LOCAL_DEVICE || scope == ORC_SCOPE_GLOBAL_DEVICE;
    const int n_blocks = (scope == ORC_SCOPE_LOCAL || scope == ORC_SCOPE_LOCAL_DEVICE) ? G : 1;
    const int seg_tokens = N / n_blocks;
    const int span = per_device ? E / G : 1; /* experts that share one budget */
    int cap;
    if (mode == ORC_MODE_NONE)
        cap = seg_tokens * span;
    else
        cap = per_device ? orc_device_budget(gamma, seg_tokens, k, E, span) : orc_capacity(gamma, seg_tokens, k, E);
    int64_t kept = 0;
    const size_t room = (size_t)(seg_tokens > 0 ? seg_tokens : 1) * (size_t)span;
    orc_cand_t* list = (orc_cand_t*)malloc(sizeof(orc_cand_t) * room);
    memset(keep, 0, (size_t)N * E);
    for (int b = 0; b < n_blocks; ++b) {
        for (int e0 = 0; e0 < E; e0 += span) {
            /* the candidates that compete for this budget: one expert, or all experts of one device */
            int n = 0;
            for (int e = e0; e < e0 + span; ++e) {
                for (int t = b * seg_tokens; t < (b + 1) * seg_tokens; ++t) {
                    if (!cand[(size_t)t * E + e]) continue;
                    list[n].cls = token_class ? (token_class[t] & 3) : 0;
                    list[n].expert = e;
                    list[n].token = t;
                    list[n].value = orc_importance(scores, E, t, e, metric, seed);
                    ++n;
                }
            }
            qsort(list, (size_t)n, sizeof(orc_cand_t), orc_cand_cmp);
            const int n_keep = n < cap ? n : cap;
            for (int i = 0; i < n_keep; ++i) keep[(size_t)list[i].token * E + list[i].expert] = 1;
            kept += n_keep;
        }
    }
    free(list);
    return kept;
}

/* ---------------------------------------------------------------------------
 * At most k experts per token after the drop (Sec. 4 "Expanded Drop" and the appendix
 * "Maximum Number of Selected Experts", the "w/ max" rows of its table): with k+m
 * candidates a token may survive at more than k experts; the constrained variant retains
 * the k surviving experts with the highest gating score (equal scores: lower expert id)
 * and discards the token's other pairs.  Places freed at an expert are not handed to
 * tokens that expert dropped earlier (one round of selection and dropping, as the paper
 * argues against repeated rounds).  keep is updated in place; returns the pairs removed.
 * ------------------------------------------------------------------------- */
int64_t orc_limit_experts(const float* scores, int N, int E, int k, uint8_t* keep) {
    int64_t removed = 0;
    for (int t = 0; t < N; ++t) {
        int n_kept = 0;
        for (int e = 0; e < E; ++e) n_kept += keep[(size_t)t * E + e];
        while (n_kept > k) {
            /* discard the surviving expert with the lowest score; among equal scores the highest id */
            int worst = -1;
            for (int e = 0; e < E; ++e) {
                if (!keep[(size_t)t * E + e]) continue;
                if (worst < 0 || scores[(size_t)t * E + e] <= scores[(size_t)t * E + worst]) worst = e;
            }
            keep[(size_t)t * E + worst] = 0;
            --n_kept;
            ++removed;
        }
    }
    return removed;
}

/* ---------------------------------------------------------------------------
 * Dispatch plan: the kept pairs written as the permutation the layer executes
 * ("permutation" stage of Sec. 5.1's latency breakdown).  Rows are expert-major and
 * ascending in token inside an expert; row_weight is the un-renormalised softmax
 * score of the pair (final_scores of Alg. 1); pair_row[t, slot] is the row of the
 * token's slot-th candidate expert (candidates in ascending expert id), -1 if that
 * pair was dropped or the slot is unused.  seg_count[b,e] counts kept pairs of
 * expert e among the tokens of device block b (n_blocks = G for LOCAL scope, else 1).
 * Returns P, the number of rows.
 * ------------------------------------------------------------------------- */
int64_t orc_build_plan(const float* scores, const uint8_t* cand, const uint8_t* keep, int N, int E, int S,
                       int n_blocks, int32_t* expert_count, int32_t* seg_count, int32_t* expert_offset,
                       int32_t* row_token, float* row_weight, int32_t* pair_row) {
    const int seg_tokens = N / n_blocks;
    int64_t r = 0;
    for (int i = 0; i < N * S; ++i) pair_row[i] = -1;
    for (int i = 0; i < n_blocks * E; ++i) seg_count[i] = 0;
    for (int e = 0; e < E; ++e) {
        expert_offset[e] = (int32_t)r;
        for (int t = 0; t < N; ++t) {
            if (!keep[(size_t)t * E + e]) continue;
            int slot = 0;
            for (int e2 = 0; e2 < e; ++e2) slot += cand[(size_t)t * E + e2];
            row_token[r] = t;
            row_weight[r] = scores[(size_t)t * E + e];
            pair_row[(size_t)t * S + slot] = (int32_t)r;
            seg_count[(t / seg_tokens) * E + e] += 1;
            ++r;
        }
        expert_count[e] = (int32_t)r - expert_offset[e];
    }
    expert_offset[E] = (int32_t)r;
    return r;
}

/* ---------------------------------------------------------------------------
 * Expert function and layer output, Eq. (2): y = sum_{i in K} G(x)_i * E_i(x), over the
 * pairs that survive the drop, with the masked un-renormalised scores as weights
 * (final_scores of Alg. 1).  The paper does not define E_i; the workloads fix it as a
 * bias-free SwiGLU FFN:  E_i(v) = W_down ( silu(W_gate v) * (W_up v) ),
 * silu(a) = a / (1 + exp(-a)).
 * Everything is accumulated in fp64 from the stored (fp32 / bf16-valued) inputs with
 * no intermediate rounding.  A token with no surviving pair gets y = 0.
 *
 * w_gate[e], w_up[e] are [h,d], w_down[e] is [d,h]; a NULL entry is allowed for an
 * expert no listed token uses (returns -1 if it is needed).  `token_list` selects the
 * tokens to compute (NULL: all N); y is [n_list, d].
 * ------------------------------------------------------------------------- */
static void orc_expert_ffn(const float* v, const float* wg, const float* wu, const float* wd, int d, int h,
                           double* act, double* out) {
    for (int j = 0; j < h; ++j) {
        double g = 0.0, u = 0.0;
        for (int i = 0; i < d; ++i) {
            g += (double)wg[(size_t)j * d + i] * (double)v[i];
            u += (double)wu[(size_t)j * d + i] * (double)v[i];
        }
        act[j] = g / (1.0 + exp(-g)) * u;
    }
    for (int i = 0; i < d; ++i) {
        double o = 0.0;
        for (int j = 0; j < h; ++j) o += (double)wd[(size_t)i * h + j] * act[j];
        out[i] = o;
    }
}

int orc_layer_output(const float* x, const float* scores, const uint8_t* keep, const float* const* w_gate,
                     const float* const* w_up, const float* const* w_down, int N, int d, int E, int h,
                     const int32_t* token_list, int n_list, double* y) {
    int status = 0;
    if (!token_list) n_list = N;
#pragma omp parallel
    {
        double* act = (double*)malloc(sizeof(double) * (size_t)h);
        double* out = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (int q = 0; q < n_list; ++q) {
            const int t = token_list ? token_list[q] : q;
            double* yt = y + (size_t)q * d;
            for (int i = 0; i < d; ++i) yt[i] = 0.0;
            for (int e = 0; e < E; ++e) {
                if (!keep[(size_t)t * E + e]) continue;
                if (!w_gate[e] || !w_up[e] || !w_down[e]) {
#pragma omp atomic write
                    status = -1;
                    continue;
                }
                orc_expert_ffn(x + (size_t)t * d, w_gate[e], w_up[e], w_down[e], d, h, act, out);
                const double g = (double)scores[(size_t)t * E + e];
                for (int i = 0; i < d; ++i) yt[i] += g * out[i];
            }
        }
        free(act);
        free(out);
    }
    return status;
}
