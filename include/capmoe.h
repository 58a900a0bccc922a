/*
 * capmoe - capacity-aware Mixture-of-Experts layer forward on one AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Capacity-Aware Inference: Mitigating the Straggler Effect in
 * Mixture of Experts" (arXiv 2503.05066): router -> softmax -> top-k (Eq. 1), expert capacity
 * C = gamma * N_bar (Sec. 4), score-ranked Token Drop (Eqs. 8-10, Alg. 1) or Expanded Drop
 * (Sec. 4 "Expanded Drop", Alg. 2), permutation, expert FFNs and the weighted sum (Eq. 2).
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers (HIP global memory) unless marked "host".  The caller
 *     owns every buffer; the library allocates nothing, frees nothing and keeps no pointer after
 *     the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work; they never synchronise.  Work of one layer must be enqueued on one stream, in the
 *     order route_topk, capacity_drop, dispatch, grouped_ffn, combine.
 *   - Matrices are row-major and dense (no strides).  Indices are int32.
 *   - Every function returns a moe_status_t.  Arguments are validated on the host before any
 *     launch; on a non-zero status nothing was enqueued.  MOE_ERR_HIP reports a failed launch.
 *   - `workspace` is scratch device memory of at least the size moe_query reports, 256-byte
 *     aligned, reusable between calls (its content has no meaning after a call completes).
 *   - Calls act on the current device.  The library holds no state of a call; what it remembers is per
 *     device and written atomically (which kernel attributes it has set there, the compute-unit count, the
 *     address of the built-in buffer of moe_route_topk_static), so any host thread may call on any device.
 *
 * Simulated expert parallelism: with G = device_groups, token t lives on device t / (N/G) and
 * device b hosts experts [b*E/G, (b+1)*E/G) (data parallel = expert parallel, as in the paper's
 * deployment, Sec. 5.1).  N and E must be multiples of G.
 */
#ifndef CAPMOE_H
#define CAPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,         /* null pointer, size out of range, N or E not a multiple of G   */
    MOE_ERR_UNSUPPORTED = 2,         /* valid but not implemented (shape granularity, dtype)          */
    MOE_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below what moe_query reports                  */
    MOE_ERR_HIP = 4,                 /* the HIP runtime refused a launch                              */
    MOE_ERR_SCRATCH_LIMIT = 5        /* moe_route_topk_static: the problem needs more scratch memory
                                        than the library's built-in buffer holds                      */
} moe_status_t;

enum { MOE_MODE_NONE = 0, MOE_MODE_TOKEN_DROP = 1, MOE_MODE_EXPANDED_DROP = 2 };
/* Where a capacity constraint applies: per expert (Sec. 4) or per device (Sec. 5.2, "Advanced Variant:
 * Device-Level Capacity-Aware Inference"), over the tokens of one device (LOCAL) or over all tokens */
enum { MOE_SCOPE_LOCAL = 0, MOE_SCOPE_GLOBAL = 1, MOE_SCOPE_LOCAL_DEVICE = 2, MOE_SCOPE_GLOBAL_DEVICE = 3 };
enum { MOE_DTYPE_F32 = 0, MOE_DTYPE_BF16 = 1 };
/* What ranks the candidates of an overflowed expert (Sec. 4, list of metrics) */
enum { MOE_METRIC_SCORE = 0, MOE_METRIC_ORDER = 1, MOE_METRIC_REVERSE_ORDER = 2, MOE_METRIC_RANDOM = 3 };

/* Shape and policy of one layer call (host memory, plain data). */
typedef struct {
    int32_t n_tokens;       /* N                                                                     */
    int32_t d_model;        /* d                                                                     */
    int32_t n_experts;      /* E, at most 256                                                        */
    int32_t top_k;          /* k, 1 <= k <= min(E, 64)                                               */
    int32_t d_hidden;       /* h, SwiGLU hidden width                                                */
    int32_t device_groups;  /* G >= 1 simulated devices                                              */
    int32_t mode;           /* MOE_MODE_*: plain top-k, Token Drop (Alg. 1), Expanded Drop (Alg. 2)  */
    int32_t capacity_scope; /* MOE_SCOPE_LOCAL: capacity per (device's tokens, expert), with
                               N/G tokens in the capacity formula (Sec. 4: constraints are applied
                               within each local device).  MOE_SCOPE_GLOBAL: per expert over all N.
                               MOE_SCOPE_LOCAL_DEVICE / MOE_SCOPE_GLOBAL_DEVICE: one budget for the E/G
                               experts of a device, N_1 + ... + N_nl <= n_l * gamma * N_bar (Sec. 5.2): all
                               candidate pairs of the device's experts are ranked together (equal rank:
                               lower token, then lower expert id); the paper states the constraint, the
                               ranking rule is this library's reading.                               */
    double gamma;           /* capacity factor, >= 0 or +infinity (Sec. 4)                           */
    int32_t dtype;          /* MOE_DTYPE_*: type of x, expert weights, xp, yp, y.  The router
                               (logits, softmax, scores) is always fp32.                             */
    int32_t metric;         /* MOE_METRIC_*: SCORE keeps the highest gating scores (the paper's choice),
                               ORDER the earliest tokens, REVERSE_ORDER the latest, RANDOM a uniform
                               draw per pair; 0 = SCORE                                              */
    int32_t overselect;     /* m >= 0: every token offers itself to its top-(k+m) experts instead of its
                               top-k (over-selection ratio m of Sec. 5.2, "Effectiveness of Expanded
                               Drop"; m = 2k, 3k in the appendix "Maximum Number of Selected Experts").
                               The capacity keeps using k.  k + m <= min(E, 64).  topk_idx and
                               topk_score are then [N, k+m].  0 = the plain method                  */
    int32_t max_experts;    /* 1 = "w/ max" of that appendix: after the drop a token keeps at most k of
                               its surviving experts, those with the highest gating score (equal
                               scores: lower expert id); places this frees are not refilled.
                               0 = no limit (the paper's choice)                                     */
} moe_desc_t;

const char* moe_status_string(int status);

/*
 * Static sizes of a layer call (host-only, launches nothing).
 *   cap             capacity of one segment: min(Ns, trunc(gamma * (Ns*k) / E)), Ns = N (GLOBAL) or
 *                   N/G (LOCAL); Ns for MOE_MODE_NONE or gamma = +inf.  (Sec. 4; Alg. 1)
 *                   Device scopes: the device budget min(Ns*E/G, trunc(gamma * (Ns*k*E/G) / E)).
 *   slots_per_token S = k + overselect, plus E/G for Expanded Drop (a token may keep up to k+m experts,
 *                   Sec. 4)
 *   max_rows        P_max, an upper bound on surviving token-expert pairs: size xp, yp, row_token,
 *                   row_weight for this many rows
 *   workspace_bytes enough for any single call of this descriptor
 * Any output pointer may be NULL.
 */
int moe_query(const moe_desc_t* desc, int32_t* cap, int32_t* slots_per_token, int64_t* max_rows,
              size_t* workspace_bytes);

/*
 * Router, softmax and top-k: K = TopK(Softmax(G(x)), k), Eq. (1).
 *   x            [N,d] in desc->dtype (ignored when use_given_logits != 0)
 *   w_router     [E,d] fp32;  bias [E] fp32 or NULL        (ignored when use_given_logits != 0)
 *   logits       [N,E] fp32: written, or read as input when use_given_logits != 0
 *   scores       [N,E] fp32 out: softmax over experts, computed in fp32 by a fixed operation
 *                sequence (max, exp by range reduction and a degree-7 polynomial, ascending sum,
 *                IEEE division), so equal logits give bit-equal scores
 *   topk_idx     [N,k'] int32 out, topk_score [N,k'] fp32 out, k' = k + desc->overselect: best first;
 *                equal scores go to the lower expert id
 * Logits must be finite.
 */
int moe_route_topk(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                   int use_given_logits, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_route_topk for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus the workspace, same
 * results bit for bit.  The split-K partial sums of the router GEMM go to a buffer built into the library
 * (16 MiB of device memory per GPU, held from the moment the library is loaded there until the process
 * ends); the call allocates and frees nothing.
 *   - A descriptor whose router needs more than 16 MiB of partial sums (moe_query reports more for the
 *     routing step) is refused with MOE_ERR_SCRATCH_LIMIT before anything is enqueued.  All five
 *     workloads of the benchmark fit (at most 8 MiB).
 *   - The buffer belongs to the device that is current at the call.  Every call on a GPU shares that
 *     GPU's buffer: two calls that overlap on one GPU (different streams, different threads) race; calls
 *     on one stream are safe, and nothing in the buffer needs clearing between calls (every partial sum
 *     that is read was written by the same call).
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress), which is when the HIP
 *     runtime places the buffer in that device's memory; make that one call outside a graph capture.  No
 *     later call changes the amount of free device memory.
 */
int moe_route_topk_static(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                          int use_given_logits, float* logits, float* scores, int32_t* topk_idx,
                          float* topk_score, void* stream);

/*
 * Capacity enforcement: Token Drop (Eqs. 8-10, Alg. 1) or Expanded Drop (Alg. 2), or none.
 * Candidates of token t: the k + overselect experts listed in topk_idx; Expanded Drop adds the E/G
 * experts of the token's own device.  In every capacity segment (expert, or device-block x expert for LOCAL scope) the `cap`
 * candidates that rank highest under desc->metric (the gating score by default) are kept; equal rank
 * goes to the lower token index.
 * Outputs (the dispatch plan; B = G for the LOCAL scopes, 1 for the GLOBAL ones):
 *   expert_count  [E]     kept pairs per expert
 *   seg_count     [B,E]   kept pairs per (device block, expert)
 *   expert_offset [E+1]   exclusive prefix sum of expert_count; expert_offset[E] = P
 *   row_token     [P_max] token of each row; rows are expert-major, ascending token inside an expert
 *   row_weight    [P_max] softmax score of the pair (un-renormalised; final_scores of Alg. 1)
 *   pair_row      [N,S]   row of the token's slot-th candidate expert (candidates in ascending
 *                         expert id), or -1 if dropped / slot unused
 * Entries of row_token / row_weight at or beyond P are left untouched.
 * Preconditions the call does not check (they hold for the outputs of moe_route_topk): every score is the
 * softmax of Eq. (1), 0 <= s <= 1 and not NaN (candidates are ranked on the bit patterns of their scores, which
 * order like the values only for non-negative numbers, and the two top bits of a key hold the token class); every
 * row of topk_idx holds distinct expert ids in [0, E).  scores, topk_idx and pair_row must be 16-byte aligned
 * (checked: MOE_ERR_INVALID_ARG).
 */
int moe_capacity_drop(const moe_desc_t* desc, const float* scores, const int32_t* topk_idx,
                      int32_t* expert_count, int32_t* seg_count, int32_t* expert_offset, int32_t* row_token,
                      float* row_weight, int32_t* pair_row, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * moe_capacity_drop with the two optional inputs of the other drop policies:
 *   token_class [N] uint8 or NULL  the multimodal strategies (Sec. "Extension to Multimodal Mixture of
 *              Experts"): a candidate of a lower class (0..3) is dropped before any candidate of a
 *              higher class, whatever the metric says; "Image First" = image tokens 0, text tokens 1;
 *              NULL = "Uniform" (one class).
 *   seed       MOE_METRIC_RANDOM draws, for the pair (t, e), the 29 high bits of a 32-bit integer hash
 *              of the counter t*E + e offset by seed * 0x9E3779B9 (x ^= x>>16; x *= 0x7FEB352D;
 *              x ^= x>>15; x *= 0x846CA68B; x ^= x>>16): a counter-based generator, reproducible
 *              anywhere.  Ignored by the other metrics.
 * Equal rank goes to the lower token index.  row_weight is the gating score whatever ranks the tokens.
 */
int moe_capacity_drop_ranked(const moe_desc_t* desc, const float* scores, const int32_t* topk_idx,
                             const uint8_t* token_class, uint32_t seed, int32_t* expert_count, int32_t* seg_count,
                             int32_t* expert_offset, int32_t* row_token, float* row_weight, int32_t* pair_row,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Permutation (the "permutation" stage of the latency breakdown, Sec. 5.1):
 * xp[r,:] = x[row_token[r],:] for r < P = expert_offset[E].  xp is [P_max,d]; rows >= P untouched.
 */
int moe_dispatch(const moe_desc_t* desc, const void* x, const int32_t* expert_offset, const int32_t* row_token,
                 void* xp, void* stream);

/*
 * Expert computation E_i(x) of Eq. (2) on the permuted rows.  The paper leaves E_i open; here it
 * is a bias-free SwiGLU FFN: yp[r,:] = W_down[e] ( silu(W_gate[e] xp[r,:]) * (W_up[e] xp[r,:]) ) for
 * the rows r of expert e, i.e. expert_offset[e] <= r < expert_offset[e+1].
 *   w_gate, w_up [E,h,d], w_down [E,d,h] in desc->dtype.  bf16: fp32 accumulation on the matrix
 *   cores, the hidden activation is rounded to bf16 once; d and h must be multiples of 128.
 *   yp [P_max,d]; rows >= P untouched.
 */
int moe_grouped_ffn(const moe_desc_t* desc, const void* xp, const int32_t* expert_offset, const void* w_gate,
                    const void* w_up, const void* w_down, void* yp, void* workspace, size_t workspace_bytes,
                    void* stream);

/*
 * moe_dispatch followed by moe_grouped_ffn in one call, without materialising xp: the first GEMM
 * fetches row r of the plan from x[row_token[r],:] directly (same arithmetic, bit-identical yp).
 *   x [N,d] in desc->dtype, row_token [P_max] and expert_offset [E+1] from moe_capacity_drop.
 *   bf16: x must be smaller than 4 GiB (N*d < 2^31), else MOE_ERR_UNSUPPORTED (use the two separate calls).
 */
int moe_dispatch_ffn(const moe_desc_t* desc, const void* x, const int32_t* expert_offset, const int32_t* row_token,
                     const void* w_gate, const void* w_up, const void* w_down, void* yp, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * Weighted sum of Eq. (2) over the surviving pairs: y[t,:] = sum_slots row_weight[r] * yp[r,:],
 * r = pair_row[t,slot] >= 0, slots in ascending order (= ascending expert id), accumulated in
 * fp32.  A token with no surviving pair gets y[t,:] = 0.  y is [N,d].
 */
int moe_combine(const moe_desc_t* desc, const void* yp, const float* row_weight, const int32_t* pair_row, void* y,
                void* stream);

/*
 * The whole layer in one call: moe_route_topk, moe_capacity_drop_ranked, moe_dispatch_ffn and moe_combine
 * enqueued in that order on `stream` (Eq. 1, Alg. 1 / Alg. 2, Eq. 2).  Same buffers, same results bit for
 * bit as the separate calls; xp is not materialised.  token_class may be NULL; logits, scores, the top-k
 * lists and the plan are outputs the caller may inspect afterwards.  Nothing is enqueued unless every
 * argument check of the four calls passes.
 */
int moe_layer_forward(const moe_desc_t* desc, const void* x, const float* w_router, const float* bias,
                      const void* w_gate, const void* w_up, const void* w_down, const uint8_t* token_class,
                      uint32_t seed, float* logits, float* scores, int32_t* topk_idx, float* topk_score,
                      int32_t* expert_count, int32_t* seg_count, int32_t* expert_offset, int32_t* row_token,
                      float* row_weight, int32_t* pair_row, void* yp, void* y, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * Profiling hook (instrumentation, not part of the method).  The table is the caller's (host memory); the
 * library keeps only a pointer to it, per host thread, between moe_profile_attach(table) and
 * moe_profile_attach(NULL).  While a table is attached to the calling thread, every launch of kernel id k by
 * that thread increments launches[k] and, where start[k] / stop[k] are not NULL, records those hipEvent_t
 * (passed as void*) before / after the launch on the launch stream: hipEventElapsedTime(start, stop) is then
 * that launch's duration, and launches[k] == 0 tells that the call sequence never ran the kernel.
 */
enum {
    MOE_KERNEL_ROUTER_LOGITS = 0,
    MOE_KERNEL_SOFTMAX_TOPK = 1,
    MOE_KERNEL_DROP_PREPARE = 2,
    MOE_KERNEL_DROP_SELECT = 3, /* also the single kernel that replaces prepare, select and emit on small problems */
    MOE_KERNEL_DROP_EMIT = 4,
    MOE_KERNEL_DISPATCH = 5,
    MOE_KERNEL_FFN_SCHEDULE = 6,
    MOE_KERNEL_FFN_GATE_UP = 7,
    MOE_KERNEL_FFN_DOWN = 8,
    MOE_KERNEL_COMBINE = 9,
    MOE_KERNEL_DROP_LIMIT = 10, /* only launched with max_experts */
    MOE_KERNEL_COUNT = 11
};
typedef struct {
    void* start[MOE_KERNEL_COUNT];
    void* stop[MOE_KERNEL_COUNT];
    int64_t launches[MOE_KERNEL_COUNT];
} moe_profile_t;
int moe_profile_attach(moe_profile_t* table);

/*
 * What the tile schedule of the expert GEMMs decides for a plan with the given rows per expert (diagnostic; the
 * library runs the same code on the device when it builds the schedule, here it runs on the host and launches
 * nothing).  Lets a caller or a test see which launch form a workload gets.
 *   expert_count    host [E]: rows per expert of the plan (their sum at most max_rows of moe_query)
 *   compute_units   compute units of the GPU the answer is for (256 on MI355X; a multiple of 8)
 *   tiles           host [2], out: full-height (256-row) tiles, short (64-row) tiles
 *   header          host [2][8], out: for the gate/up GEMM, then the down GEMM:
 *                   [0] big work items per XCD that are cut along K, [1] units per such item,
 *                   [2], [3] the same for the short items, [4] 1 if the GEMM walks the joint tile list,
 *                   [5] work items at the end of that list that the XCDs share out by a counter,
 *                   [6] big work items per XCD that run as four 64-row blocks, [7] 0.
 *                   All zero for desc->dtype == fp32, whose kernels use none of this.
 * Errors: MOE_ERR_INVALID_ARG for null pointers, negative counts, more rows than max_rows.
 */
int moe_ffn_schedule_query(const moe_desc_t* desc, const int32_t* expert_count, int compute_units, int32_t* tiles,
                           int32_t* header);

/*
 * Matrix-core ceiling probe (instrumentation, not part of the method): launches `blocks` workgroups of
 * 4 wavefronts that each repeat `iterations` times the 64 independent bf16 MFMAs (16x16x32) of one k-step of
 * the layer's big GEMM tile, on register operands.
 *   random_operands  0: operands of zeros and ones; otherwise random bf16 values in (-2, 2).  The clock the
 *                    chip holds under the loop, and so the rate, depends on how many operand bits switch.
 *   sink   device, at least blocks * 256 floats (receives checksums)
 *   flops  host, optional: floating-point operations of the launch, 2*16*16*32 per MFMA
 * The caller times the launch; flops / time is what the matrix cores sustain with no memory traffic.
 * blocks <= 65536, iterations <= 2^20.
 */
int moe_probe_mfma_bf16(int blocks, int iterations, int random_operands, float* sink, int64_t* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CAPMOE_H */
