// Capacity enforcement: Token Drop (Eqs. 8-10, Alg. 1) and Expanded Drop (Alg. 2).
//
// Three kernels, all integer work on score bit patterns (scores are >= +0, so the unsigned
// order of the bits is the order of the values):
//   1. drop_prepare   per token: candidate set (top-k, plus the experts of the token's own device
//                     for Expanded Drop) -> key = rank + 1 for candidates, 0 otherwise, written
//                     expert-major so that a capacity segment is one contiguous run.  The rank is
//                     the score's bit pattern (Score metric), the token's position (Order, Reverse
//                     Order) or a hashed draw (Random), below an optional 2-bit token class.
//   2. drop_select    per segment: the cap-th largest key by a 4-pass radix select over LDS
//                     histograms (the threshold tau of Eq. 8) and how many keys equal to it survive.
//   3. drop_emit      per segment (a block per 4096 tokens of it): ordered compaction of the survivors,
//                     which yields rows in ascending token order and gives ties at the threshold to
//                     the lower token index.
// Every kernel first pulls what it needs from global memory in one batch of independent loads
// (these kernels are latency-bound: a dependent load per loop iteration costs a microsecond each).
// Small problems with per-expert capacities run all three steps in one launch (drop_fused, below),
// the optional per-token limit adds a fourth kernel and a second emit.
#include <type_traits>

#include "common.h"
#include "schedule.h"

namespace capmoe {

constexpr int kPrepTokens = 16;  // tokens per block: small, the kernel is latency-bound and wants every CU

// The draw of MOE_METRIC_RANDOM: a 32-bit integer hash (two multiply-xorshift rounds) of the pair's
// counter, offset by the seed; the header states the same formula.
__device__ inline uint32_t pair_hash(uint32_t seed, uint32_t counter) {
    uint32_t x = counter + seed * 0x9E3779B9u;
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

// ---------------------------------------------------------------------------------------------
// 1. candidate keys, transposed
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void drop_prepare_kernel(const float* __restrict__ scores,
                                                           const int32_t* __restrict__ topk_idx,
                                                           uint32_t* __restrict__ key_t, uint8_t* __restrict__ slot_t,
                                                           int32_t* __restrict__ pair_row, int N, int E, int k, int S,
                                                           int expanded, int group_tokens, int group_experts,
                                                           int metric, int seg_tokens,
                                                           const uint8_t* __restrict__ token_class, uint32_t seed) {
    extern __shared__ uint32_t lds[];
    const int ld = E | 1;                                  // odd row pitch: conflict-free transposed reads
    uint32_t* key_s = lds;                                 // [kPrepTokens][ld] score bits, then keys
    uint8_t* slot_s = (uint8_t*)(lds + kPrepTokens * ld);  // [kPrepTokens][ld] candidate flags, then slots
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int t0 = blockIdx.x * kPrepTokens;
    const int nt = N - t0 < kPrepTokens ? N - t0 : kPrepTokens;  // tokens of this block

    for (int i = tid; i < kPrepTokens * ld; i += 256) slot_s[i] = 0;
    // the block's scores are one contiguous run of nt*E floats
    for (int i = tid; i < nt * E; i += 256) {
        const int tl = i / E, e = i - tl * E;
        key_s[tl * ld + e] = __float_as_uint(scores[(size_t)t0 * E + i]);
    }
    __syncthreads();
    for (int i = tid; i < nt * k; i += 256) slot_s[(i / k) * ld + topk_idx[(size_t)t0 * k + i]] = 1;
    if (expanded) {
        for (int i = tid; i < nt * group_experts; i += 256) {
            const int tl = i / group_experts, j = i - tl * group_experts;
            slot_s[tl * ld + ((t0 + tl) / group_tokens) * group_experts + j] = 1;
        }
    }
    __syncthreads();
    // flags -> keys and slots (slot = number of candidate experts with a lower id); a wave walks its tokens
    constexpr int kWalk = kPrepTokens / 4;
    for (int i = 0; i < kWalk; ++i) {
        const int tl = wv * kWalk + i, t = t0 + tl;
        if (tl >= nt) break;
        int base = 0;
        const uint32_t cls = token_class ? (uint32_t)(token_class[t] & 3) << 30 : 0u;
        const int local = t % seg_tokens;  // position inside the capacity segment
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            const bool c = e < E && slot_s[tl * ld + e] != 0;
            const uint64_t mask = __ballot(c);
            if (e < E) {
                // rank within the class, below 2^30: score bits (scores are in [0,1]), position, or a draw
                uint32_t rank;
                if (metric == MOE_METRIC_ORDER)
                    rank = (uint32_t)(seg_tokens - 1 - local);
                else if (metric == MOE_METRIC_REVERSE_ORDER)
                    rank = (uint32_t)local;
                else if (metric == MOE_METRIC_RANDOM)
                    rank = pair_hash(seed, (uint32_t)t * (uint32_t)E + (uint32_t)e) >> 3;
                else
                    rank = key_s[tl * ld + e];
                key_s[tl * ld + e] = c ? cls + rank + 1u : 0u;
                slot_s[tl * ld + e] = (uint8_t)(base + __popcll(mask & ((1ull << lane) - 1ull)));
            }
            base += __popcll(mask);
        }
        // slots beyond the token's candidate count stay unused
        for (int s = base + lane; s < S; s += kWave) pair_row[(size_t)t * S + s] = -1;
    }
    __syncthreads();
    // transposed write: a wave writes the block's consecutive tokens of 64 / kPrepTokens experts at a time
    constexpr int kRows = kWave / kPrepTokens;
    const int tl = lane % kPrepTokens;
    for (int e = wv * kRows + lane / kPrepTokens; e < E; e += 4 * kRows) {
        if (tl < nt) {
            key_t[(size_t)e * N + t0 + tl] = key_s[tl * ld + e];
            slot_t[(size_t)e * N + t0 + tl] = slot_s[tl * ld + e];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// block-wide helpers (NT threads, a multiple of the wave width)
// ---------------------------------------------------------------------------------------------
template <int NT>
__device__ inline int block_sum(int v, int* red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    int total = 0;
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) total += red[w];
    return total;
}
__device__ inline int block_sum_256(int v, int* red) { return block_sum<256>(v, red); }

// exclusive prefix sum of v over the block's threads; *total gets the block sum
template <int NT>
__device__ inline int block_exclusive_scan(int v, int* red, int* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += o;
    }
    __syncthreads();
    if (lane == 63) red[wv] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) {
        if (w < wv) before += red[w];
        all += red[w];
    }
    *total = all;
    return before + incl - v;
}
__device__ inline int block_exclusive_scan_256(int v, int* red, int* total) {
    return block_exclusive_scan<256>(v, red, total);
}

// ---------------------------------------------------------------------------------------------
// 2. threshold per segment
// ---------------------------------------------------------------------------------------------
constexpr int kSelectCache = 32768;  // keys of a segment kept in LDS (up to 128 KB); longer segments re-read L2

// One block per capacity segment: `span` experts (1, or the E/G experts of a device when the
// capacity is a device budget) over seg_tokens tokens.  The keys of expert e0+r form run r.
// Outputs, per (block, expert): the threshold, how many keys equal to it survive, the kept count.
// Several experts under one budget share the threshold; the keys equal to it are granted to the
// lower tokens first and, inside a token, to the lower expert ids.
// NT threads: 256 for short segments, 1024 for long ones (a segment is one block's work, and its
// passes over the keys are chains of load latencies that only more loads in flight shorten).
// VEC keys per load: 4 when every run starts on a 16-byte boundary (N and seg_tokens multiples of 4).
template <int NT, int VEC>
__global__ __launch_bounds__(NT) void drop_select_kernel(const uint32_t* __restrict__ key_t,
                                                          uint32_t* __restrict__ seg_tau,
                                                          int32_t* __restrict__ seg_need,
                                                          int32_t* __restrict__ seg_count, int N, int E, int seg_tokens,
                                                          int span, int cap) {
    extern __shared__ __attribute__((aligned(16))) uint32_t cache[];
    __shared__ int hist[256];
    __shared__ int gt_s[kMaxExperts], eq_s[kMaxExperts];
    __shared__ int red[NT / kWave];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_rem;
    const int groups = E / span;
    const int b = blockIdx.x / groups, e0 = (blockIdx.x - b * groups) * span;
    const uint32_t* keys = key_t + (size_t)e0 * N + (size_t)b * seg_tokens;  // run r starts at keys + r*N
    const int tid = threadIdx.x;
    const int n_keys = span * seg_tokens;
    const bool cached = n_keys <= kSelectCache;

    // Every pass walks all keys of the segment, key i = run i / seg_tokens, token i % seg_tokens: a thread
    // requests kBatch loads of VEC keys before it uses any, then calls f(run, token, key) key by key (in
    // ascending i per thread).
    constexpr int kBatch = NT > 256 ? 16 : 8;
    struct alignas(4 * VEC) KeyVec {
        uint32_t c[VEC];
    };
    auto for_each_key = [&](bool from_cache, auto&& f) {
        for (int i0 = tid * VEC; i0 < n_keys; i0 += NT * VEC * kBatch) {
            KeyVec kx[kBatch];
            int run[kBatch], tok[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + NT * VEC * u;  // VEC divides seg_tokens: the keys of a load share a run
                run[u] = span == 1 ? 0 : i / seg_tokens;  // (a division is as much work as four keys)
                tok[u] = i - run[u] * seg_tokens;
                if (i >= n_keys) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) kx[u].c[c] = 0u;
                } else if (from_cache) {
                    kx[u] = *(const KeyVec*)(cache + i);
                } else {
                    kx[u] = *(const KeyVec*)(keys + (size_t)run[u] * N + tok[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (i0 + NT * VEC * u < n_keys) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) f(run[u], tok[u] + c, kx[u].c[c]);
                }
        }
    };

    // load the keys; the histogram of their top byte (the first radix pass) is taken on the way
    if (tid < 256) hist[tid] = 0;
    for (int r = tid; r < span; r += NT) gt_s[r] = eq_s[r] = 0;
    __syncthreads();
    int mine = 0;
    for_each_key(false, [&](int r, int tl, uint32_t key) {
        if (cached) cache[r * seg_tokens + tl] = key;
        if (key != 0u) {  // non-candidates (key 0) never matter
            ++mine;
            atomicAdd(&hist[key >> 24], 1);
        }
    });
    const int n_cand = block_sum<NT>(mine, red);  // its barriers also order the LDS writes before the reads

    // threshold: keys above tau are kept, `rem` of the keys equal to tau are kept
    uint32_t tau = 0;  // every candidate (key >= 1) passes
    int rem = 0;
    if (cap == 0) {
        tau = 0xffffffffu;  // nothing passes
    } else if (n_cand > cap) {
        // cap-th largest key, most significant byte first
        uint32_t prefix = 0;
        rem = cap;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (shift != 24) {
                if (tid < 256) hist[tid] = 0;
                __syncthreads();
                const uint32_t hi_mask = 0xffffffffu << (shift + 8);
                auto count_digit = [&](int, int, uint32_t key) {
                    if (key != 0u && (key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
                };
                for_each_key(cached, count_digit);
                __syncthreads();
            }
            // thread i < 256 owns digit 255 - i: an exclusive scan over threads counts the keys with a larger
            // digit; the digit where that count first reaches `rem` holds the cap-th key
            const int mine_d = 255 - tid;
            const int h = tid < 256 ? hist[mine_d] : 0;
            int total;
            const int above = block_exclusive_scan<NT>(h, red, &total);
            if (tid < 256 && above + h >= rem && above < rem) {  // exactly one thread
                sh_prefix = prefix | ((uint32_t)mine_d << shift);
                sh_rem = rem - above;
            }
            __syncthreads();
            prefix = sh_prefix;
            rem = sh_rem;
        }
        tau = prefix;
    }
    if (span == 1) {  // one expert: the counts follow from the selection itself
        if (tid == 0) {
            const int seg = b * E + e0;
            seg_tau[seg] = tau;
            seg_need[seg] = rem;
            seg_count[seg] = cap == 0 ? 0 : (n_cand > cap ? cap : n_cand);
        }
        return;
    }
    // per expert: keys above the threshold and keys equal to it (a thread's keys change run rarely)
    auto count_runs = [&](int tie_token, int tie_run) {
        int run = -1, gt = 0, eq = 0;
        for_each_key(cached, [&](int r, int tl, uint32_t key) {
            if (r != run) {
                if (gt) atomicAdd(&gt_s[run], gt);
                if (eq) atomicAdd(&eq_s[run], eq);
                run = r;
                gt = eq = 0;
            }
            gt += key > tau;
            eq += key == tau && key != 0u && (tl < tie_token || (tl == tie_token && r <= tie_run));
        });
        if (gt) atomicAdd(&gt_s[run], gt);
        if (eq) atomicAdd(&eq_s[run], eq);
    };
    count_runs(seg_tokens, span);  // every key equal to the threshold
    __syncthreads();
    int eq_total = 0;
    for (int r = 0; r < span; ++r) eq_total += eq_s[r];
    if (eq_total > rem) {
        // More keys equal the threshold than the budget has room for: they are granted in
        // (token, expert) order.  A thread owns a run of consecutive tokens; the thread in whose
        // run the budget ends finds the last granted pair (token tie_token, expert run tie_run).
        __shared__ int sh_tie_token, sh_tie_run;
        const int per = (seg_tokens + NT - 1) / NT;
        const int tb = tid * per < seg_tokens ? tid * per : seg_tokens;
        const int te = tb + per < seg_tokens ? tb + per : seg_tokens;
        auto key_at = [&](int r, int tl) { return cached ? cache[r * seg_tokens + tl] : keys[(size_t)r * N + tl]; };
        int c = 0;
        for (int tl = tb; tl < te; ++tl)
            for (int r = 0; r < span; ++r) c += key_at(r, tl) == tau;
        int total;
        const int before = block_exclusive_scan<NT>(c, red, &total);
        if (before < rem && rem <= before + c) {  // exactly one thread: 1 <= rem < eq_total = total
            int left = rem - before;
            for (int tl = tb; tl < te && left > 0; ++tl)
                for (int r = 0; r < span && left > 0; ++r)
                    if (key_at(r, tl) == tau && --left == 0) {
                        sh_tie_token = tl;
                        sh_tie_run = r;
                    }
        }
        __syncthreads();
        const int tie_token = sh_tie_token, tie_run = sh_tie_run;
        for (int r = tid; r < span; r += NT) gt_s[r] = eq_s[r] = 0;
        __syncthreads();
        count_runs(tie_token, tie_run);
        __syncthreads();
    }
    if (tid < span) {
        const int seg = b * E + e0 + tid;
        seg_tau[seg] = tau;
        seg_need[seg] = eq_s[tid];  // inside an expert the granted keys are its first ones in token order
        seg_count[seg] = gt_s[tid] + eq_s[tid];
    }
}

// ---------------------------------------------------------------------------------------------
// The tile schedule of the expert GEMMs, built by the drop itself
// ---------------------------------------------------------------------------------------------
// One block of the kernel that finishes the plan adds up every segment's kept count anyway (it needs its own
// first row).  When the whole layer is enqueued by one call, that block also turns the per-expert totals into
// row offsets (in LDS) and builds the tile lists of the expert GEMMs from them, so that no kernel has to be
// launched between the plan and the first GEMM just to read expert_offset back.
// tot[e]: rows of expert e (complete, block-visible); off: kMaxExperts + 1 words of LDS.  Called by the whole
// block after a barrier; its first wave does the work.
__device__ inline void build_schedule_from_totals(const int* tot, int* off, const FfnScheduleArgs& a) {
    if (threadIdx.x >= kWave) return;
    const int lane = threadIdx.x;
    int base = 0;
#pragma unroll
    for (int c = 0; c < kMaxExperts / kWave; ++c) {
        const int e = c * kWave + lane;
        const int v = e < a.E ? tot[e] : 0;
        int incl = v;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        if (e < a.E) off[e] = base + incl - v;
        base += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) off[a.E] = base;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // LDS operations of one wave complete in order: the offsets are there
    build_ffn_schedule(off, a);
}

// ---------------------------------------------------------------------------------------------
// 3. ordered compaction
// ---------------------------------------------------------------------------------------------
constexpr int kEmitRun = 16;                // consecutive tokens per thread
constexpr int kEmitChunk = 256 * kEmitRun;  // tokens per pass of the block

__global__ __launch_bounds__(256) void drop_emit_kernel(const float* __restrict__ scores,
                                                        const uint32_t* __restrict__ key_t,
                                                        const uint8_t* __restrict__ slot_t,
                                                        const uint32_t* __restrict__ seg_tau,
                                                        const int32_t* __restrict__ seg_need,
                                                        const int32_t* __restrict__ seg_count,
                                                        int32_t* __restrict__ expert_count,
                                                        int32_t* __restrict__ expert_offset,
                                                        int32_t* __restrict__ row_token, float* __restrict__ row_weight,
                                                        int32_t* __restrict__ pair_row, int N, int E, int n_blocks,
                                                        int seg_tokens, int S, int weight_from_key,
                                                        FfnScheduleArgs sched) {
    // a thread owns a run of 16 consecutive tokens; one padding word per run keeps the runs of
    // neighbouring threads on different LDS banks
    __shared__ uint32_t key_s[kEmitChunk + 256];
    __shared__ uint8_t slot_s[kEmitChunk];
    __shared__ int red[4];
    __shared__ int sched_tot[kMaxExperts], sched_off[kMaxExperts + 1];
    const bool scheduler = sched.enabled && blockIdx.x == 0;  // this block also builds the GEMMs' tile schedule
    if (scheduler) {
        for (int i = threadIdx.x; i < kMaxExperts; i += 256) sched_tot[i] = 0;
        __syncthreads();
    }
    // a block owns one chunk of kEmitChunk tokens of one segment; what the chunks before it keep it counts itself
    const int parts = seg_tokens > kEmitChunk ? (seg_tokens + kEmitChunk - 1) / kEmitChunk : 1;
    const int seg = blockIdx.x / parts;
    const int c0 = (blockIdx.x - seg * parts) * kEmitChunk;
    const int b = seg / E, e = seg - b * E;
    const int tid = threadIdx.x;

    const uint32_t* keys = key_t + (size_t)e * N + (size_t)b * seg_tokens;
    const uint8_t* slots = slot_t + (size_t)e * N + (size_t)b * seg_tokens;
    // this chunk's keys and slots: issued before anything waits
    const int n = seg_tokens - c0 < kEmitChunk ? seg_tokens - c0 : kEmitChunk;
    for (int i = tid; i < n; i += 256) {
        key_s[i + i / kEmitRun] = keys[c0 + i];
        slot_s[i] = slots[c0 + i];
    }
    // first row of this segment: all segments of lower experts, then lower blocks of this expert
    int before = 0, own = 0;
    for (int i = tid; i < n_blocks * E; i += 256) {
        const int bb = i / E, ee = i - bb * E;
        const int c = seg_count[i];
        if (ee < e || (ee == e && bb < b)) before += c;
        if (ee == e) own += c;
        if (scheduler) atomicAdd(&sched_tot[ee], c);
    }
    const int row0 = block_sum_256(before, red);
    const int own_total = block_sum_256(own, red);
    if (b == 0 && c0 == 0 && tid == 0) {
        expert_count[e] = own_total;
        expert_offset[e] = row0;
        if (e == E - 1) expert_offset[E] = row0 + own_total;
    }
    const uint32_t tau = seg_tau[seg];
    const int need = seg_need[seg];

    // the segment's tokens before this chunk: keys above the threshold, and keys equal to it (the first
    // `need` of those, in token order, are kept)
    int kept_base = 0, eq_base = 0;
    if (c0 > 0) {
        int gt = 0, eq = 0;
        if (((N | seg_tokens) & 3) == 0) {  // every run starts on a 16-byte boundary
            const uint4* k4 = (const uint4*)keys;
            for (int i0 = tid; i0 < c0 / 4; i0 += 256 * 8) {
                uint4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = i0 + 256 * u < c0 / 4 ? k4[i0 + 256 * u] : make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    gt += (v[u].x > tau) + (v[u].y > tau) + (v[u].z > tau) + (v[u].w > tau);
                    eq += (v[u].x == tau) + (v[u].y == tau) + (v[u].z == tau) + (v[u].w == tau);
                }
            }
        } else {
            for (int i0 = tid; i0 < c0; i0 += 256 * 8) {
                uint32_t v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = i0 + 256 * u < c0 ? keys[i0 + 256 * u] : 0u;
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    gt += v[u] > tau;
                    eq += v[u] == tau;
                }
            }
        }
        if (tau == 0u) eq = 0;  // key 0 is "not a candidate", never an equal key
        const int gt_total = block_sum_256(gt, red);
        eq_base = block_sum_256(eq, red);
        kept_base = gt_total + (eq_base < need ? eq_base : need);
    }
    __syncthreads();
    uint32_t kx[kEmitRun];
    int eq_cnt = 0;
#pragma unroll
    for (int j = 0; j < kEmitRun; ++j) {
        const int i = tid * kEmitRun + j;
        kx[j] = i < n ? key_s[tid * (kEmitRun + 1) + j] : 0u;
        eq_cnt += kx[j] != 0u && kx[j] == tau;
    }
    int eq_total, keep_total;
    int eq_rank = eq_base + block_exclusive_scan_256(eq_cnt, red, &eq_total);
    uint32_t keep_bits = 0;
    int keep_cnt = 0;
#pragma unroll
    for (int j = 0; j < kEmitRun; ++j) {
        const bool cand = kx[j] != 0u;
        const bool eq = cand && kx[j] == tau;
        const bool keep = cand && (kx[j] > tau || (eq && eq_rank < need));
        eq_rank += eq;
        keep_cnt += keep;
        keep_bits |= (uint32_t)keep << j;
    }
    int pos = row0 + kept_base + block_exclusive_scan_256(keep_cnt, red, &keep_total);
#pragma unroll
    for (int j = 0; j < kEmitRun; ++j) {
        if (kx[j] == 0u) continue;
        const int i = tid * kEmitRun + j;
        const int t = b * seg_tokens + c0 + i;
        const bool keep = (keep_bits >> j) & 1u;
        if (keep) {
            row_token[pos] = t;
            // the gating score, whatever ranked the pair (under the Score metric it is the key itself)
            row_weight[pos] = weight_from_key ? __uint_as_float(kx[j] - 1u) : scores[(size_t)t * E + e];
        }
        pair_row[(size_t)t * S + slot_s[i]] = keep ? pos : -1;
        pos += keep;
    }
    if (scheduler) {
        __syncthreads();
        build_schedule_from_totals(sched_tot, sched_off, sched);
    }
}

// ---------------------------------------------------------------------------------------------
// 4. at most k experts per token (optional; appendix "Maximum Number of Selected Experts")
// ---------------------------------------------------------------------------------------------
constexpr int kLimitTokens = 64;        // tokens of a block
constexpr int kLimitPitch = kLimitTokens + 1;  // words per expert row of the block's key tile in LDS

// Runs after a first emit.  For every token: its surviving pairs are listed, ranked by gating score
// (equal scores: lower expert id first), and those ranked k-th or worse are removed.  Keys of every pair
// that does not survive (dropped by capacity, or removed here) become 0, the per-segment counts are
// lowered, and thresholds are reset so that a second emit keeps exactly the non-zero keys.
// A block moves the keys of 64 tokens and all experts through LDS (the key matrix is expert-major: rows of
// consecutive tokens go in and out as whole cache lines); then a wave takes a token at a time, lanes
// over experts: the c-th candidate in ascending expert id owns slot c of the token (ballot prefix counts).
// EPL = experts per lane (E <= 64 * EPL).  Nothing in the per-token loop waits for global memory: the
// tokens' slot rows are staged in LDS beside the keys and their score rows are requested up front.
template <int EPL>
__global__ __launch_bounds__(256) void drop_limit_kernel(const float* __restrict__ scores, uint32_t* __restrict__ key_t,
                                                         int32_t* __restrict__ pair_row,
                                                         uint32_t* __restrict__ seg_tau, int32_t* __restrict__ seg_need,
                                                         int32_t* __restrict__ seg_count, int N, int E, int S, int k,
                                                         int seg_tokens, int segs) {
    extern __shared__ uint32_t tile[];            // [E][kLimitPitch] keys, then [kLimitTokens][S] rows of pair_row
    __shared__ uint2 survivors[4][256];           // per wave: (score bits, expert | slot << 16), ascending expert
    __shared__ int removed[kMaxExperts];          // pairs this block removes per expert (one global atomic each at the end)
    int32_t* rows = (int32_t*)(tile + (size_t)E * kLimitPitch);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    constexpr int kPerWave = kLimitTokens / 4;    // tokens of a wave: wv, wv + 4, ...
    const int t_first = blockIdx.x * kLimitTokens;
    const int t_last = t_first + kLimitTokens - 1 < N ? t_first + kLimitTokens - 1 : N - 1;
    float sc[kPerWave][EPL];
#pragma unroll
    for (int q = 0; q < kPerWave; ++q)
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int t = t_first + wv + 4 * q, e = lane + kWave * i;
            sc[q][i] = t < N && e < E ? scores[(size_t)t * E + e] : 0.0f;
        }
    for (int i = blockIdx.x * 256 + tid; i < segs; i += gridDim.x * 256) {
        seg_tau[i] = 0u;
        seg_need[i] = 0;
    }
    for (int e = tid; e < E; e += 256) removed[e] = 0;
    // the block's tokens lie in one capacity block when its first and last do
    const bool one_block = t_first / seg_tokens == t_last / seg_tokens;
    for (int i = tid; i < E * kLimitTokens; i += 256) {
        const int e = i / kLimitTokens, tl = i - e * kLimitTokens;
        tile[e * kLimitPitch + tl] = t_first + tl < N ? key_t[(size_t)e * N + t_first + tl] : 0u;
    }
    const int n_rows = (t_last - t_first + 1) * S;  // the block's rows of pair_row are consecutive in memory
    for (int i = tid; i < n_rows; i += 256) rows[i] = pair_row[(size_t)t_first * S + i];
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
    uint2* list = &survivors[wv][0];
#pragma unroll
    for (int q = 0; q < kPerWave; ++q) {
        const int tl = wv + 4 * q, t = t_first + tl;
        if (t >= N) break;  // wave-uniform
        int slot_base = 0, n = 0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + kWave * i;
            const uint32_t key = e < E ? tile[e * kLimitPitch + tl] : 0u;
            const bool cand = key != 0u;
            const uint64_t cand_mask = __ballot(cand);
            const int slot = slot_base + __popcll(cand_mask & below);
            slot_base += __popcll(cand_mask);
            const bool kept = cand && rows[tl * S + slot] >= 0;  // survived the capacity
            if (cand && !kept) tile[e * kLimitPitch + tl] = 0u;
            const uint64_t kept_mask = __ballot(kept);
            if (kept)
                list[n + __popcll(kept_mask & below)] =
                    make_uint2(__float_as_uint(sc[q][i]), (uint32_t)e | ((uint32_t)slot << 16));
            n += __popcll(kept_mask);
        }
        __builtin_amdgcn_wave_barrier();  // LDS operations of one wave complete in order
        if (n > k) {
            const int b = t / seg_tokens;
            for (int j = lane; j < n; j += kWave) {
                const uint2 mine = list[j];
                int better = 0;  // survivors ahead of pair j: higher score, or equal score and lower expert id
                for (int i = 0; i < n; ++i) {
                    const uint32_t si = list[i].x;  // same address in every lane
                    better += si > mine.x || (si == mine.x && i < j);
                }
                if (better >= k) {
                    const int e = (int)(mine.y & 0xffffu), sl = (int)(mine.y >> 16);
                    tile[e * kLimitPitch + tl] = 0u;
                    pair_row[(size_t)t * S + sl] = -1;
                    if (one_block)
                        atomicAdd(&removed[e], 1);
                    else
                        atomicSub(&seg_count[b * E + e], 1);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();  // the list is rewritten for the wave's next token only after these reads
    }
    __syncthreads();
    for (int i = tid; i < E * kLimitTokens; i += 256) {
        const int e = i / kLimitTokens, tl = i - e * kLimitTokens;
        if (t_first + tl < N) key_t[(size_t)e * N + t_first + tl] = tile[e * kLimitPitch + tl];
    }
    if (one_block)
        for (int e = tid; e < E; e += 256)
            if (removed[e]) atomicSub(&seg_count[(t_first / seg_tokens) * E + e], removed[e]);
}

// ---------------------------------------------------------------------------------------------
// 5. all of it in one launch, for small problems
// ---------------------------------------------------------------------------------------------
// With a few thousand tokens the three kernels above are a chain of short launches, each of which
// waits for the previous one to drain.  When every expert has its own capacity (no device budget, no
// per-token limit) a block can do the whole job for its segment alone: it needs the other segments
// only for its first output row, and their kept counts are min(candidates, capacity), which the
// block gets by counting the candidates of every segment itself from the top-k lists (read from L2
// by every block: small next to a launch as long as the lists are short).
constexpr int kFusedThreads = 1024;
constexpr int kFusedMaxTokens = 8 * kFusedThreads;  // tokens of a segment: its keys and slots live in LDS
constexpr int kFusedMaxSegs = 2048;    // capacity segments (one candidate counter each)
constexpr int kFusedCounters = 4096;   // counters in LDS: as many private copies of the segment counters as fit
constexpr long long kFusedMaxWork = 8ll << 20;  // segments x top-k list entries: above it, three launches are cheaper

// exclusive prefix sum of v over the block's NT threads; *total gets the block sum
template <int NT>
__device__ inline int fused_exclusive_scan(int v, int* red, int* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int o = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += o;
    }
    __syncthreads();
    if (lane == 63) red[wv] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) {
        const int r = red[w];
        before += w < wv ? r : 0;
        all += r;
    }
    *total = all;
    return before + incl - v;
}

// EXPANDED: Expanded Drop; ONE_BLOCK: a single capacity block (every token belongs to the block's segment
// list); VW: entries of a top-k list fetched per load (divides k).  The pass over the lists is the bulk of
// the kernel's instructions, so it is specialised.  NT: threads of the block, a segment holds at most 8 * NT
// tokens (short segments of short batches take small blocks: several per CU).
template <bool EXPANDED, bool ONE_BLOCK, int VW, int NT>
__global__ __launch_bounds__(NT) void drop_fused_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ topk_idx, const uint8_t* __restrict__ token_class,
    uint32_t seed, int32_t* __restrict__ expert_count, int32_t* __restrict__ seg_count,
    int32_t* __restrict__ expert_offset, int32_t* __restrict__ row_token, float* __restrict__ row_weight,
    int32_t* __restrict__ pair_row, int N, int E, int k, int S, int group_tokens, int group_experts, int metric,
    int seg_tokens, int n_blocks, int cap, int weight_from_key, FfnScheduleArgs sched) {
    constexpr int kWaves = NT / kWave, kMaxTok = NT * 8;
    __shared__ int sched_tot[kMaxExperts], sched_off[kMaxExperts + 1];
    const bool scheduler = sched.enabled && blockIdx.x == 0;  // this block also builds the GEMMs' tile schedule
    // a thread owns a run of consecutive tokens of the segment; one padding word per 16 keeps the runs of
    // neighbouring threads on different LDS banks
    __shared__ uint32_t key_s[kMaxTok + kMaxTok / 16];
    __shared__ uint8_t slot_s[kMaxTok];
    __shared__ int cand[kFusedCounters];
    __shared__ int hist[256];
    __shared__ int red[kWaves];
    __shared__ int red3[kWaves][3];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_rem;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int seg = blockIdx.x, b = seg / E, e = seg - b * E;
    const int segs = n_blocks * E;
    // Candidate counters: one private copy per lane of a wave where they fit (lanes that meet the same hot
    // expert in one instruction would otherwise serialise on its counter), an odd-ish pitch so that the
    // copies of one expert sit in different banks.
    const int pitch = segs + 1;
    const int copies = kFusedCounters / pitch < kWave ? kFusedCounters / pitch : kWave;  // >= 1
    auto pad = [](int i) { return i + (i >> 4); };

    for (int i = tid; i < copies * pitch; i += NT) cand[i] = 0;
    if (tid < 256) hist[tid] = 0;
    if (scheduler)
        for (int i = tid; i < kMaxExperts; i += NT) sched_tot[i] = 0;
    __syncthreads();

    // ---- one pass over the top-k lists, a thread per token: candidates of every segment (the experts of a
    // token's own device are counted later), and for the tokens of this block's segment what their list says
    // about expert e: listed experts with a lower id (bits 0-9), listed experts in all (bits 10-19), e itself
    // listed (bit 20); under Expanded Drop the experts of the token's own device do not count as listed, they
    // are candidates anyway
    {
        typedef int32_t vec_t __attribute__((ext_vector_type(VW)));
        int* mine = cand + (lane % copies) * pitch;
        constexpr int kTok = 4;        // tokens per thread and round
        constexpr int kVec = 8 / VW;   // loads per token and chunk of eight entries
        const int t_end = N;
        for (int t0 = tid; t0 < t_end; t0 += NT * kTok) {
            uint32_t info[kTok] = {0u, 0u, 0u, 0u};
            int tq[kTok];
#pragma unroll
            for (int q = 0; q < kTok; ++q) {
                const int t = t0 + NT * q;
                tq[q] = t < t_end ? t : t_end - 1;  // a token past the end re-reads the last one and is ignored below
            }
            for (int j0 = 0; j0 < k; j0 += 8) {
                vec_t x[kTok][kVec];  // independent loads, all issued before anything waits
#pragma unroll
                for (int q = 0; q < kTok; ++q)
#pragma unroll
                    for (int c = 0; c < kVec; ++c) {
                        const int j = j0 + c * VW < k ? j0 + c * VW : k - VW;  // past the list: a valid re-read
                        x[q][c] = *(const vec_t*)(topk_idx + (size_t)tq[q] * k + j);
                    }
#pragma unroll
                for (int q = 0; q < kTok; ++q) {
                    if (t0 + NT * q >= t_end) continue;
                    const int t = tq[q];
                    const int bb = ONE_BLOCK ? 0 : t / seg_tokens;
                    const int g0 = EXPANDED ? (t / group_tokens) * group_experts : 0;
                    int* row = mine + bb * E;
#pragma unroll
                    for (int c = 0; c < kVec; ++c) {
                        if (j0 + c * VW >= k) continue;  // the same for every thread
#pragma unroll
                        for (int u = 0; u < VW; ++u) {
                            const int xe = x[q][c][u];
                            const bool outside = !EXPANDED || xe < g0 || xe >= g0 + group_experts;
                            if (outside) atomicAdd(&row[xe], 1);
                            info[q] += (outside && xe < e ? 1u : 0u) + (outside ? 1u << 10 : 0u) + (xe == e ? 1u << 20 : 0u);
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kTok; ++q) {
                const int t = t0 + NT * q;
                if (t < t_end && (ONE_BLOCK || t / seg_tokens == b)) key_s[pad(t - b * seg_tokens)] = info[q];
            }
        }
    }
    __syncthreads();

    // ---- keys and slots of this block's segment ----
    {
        constexpr int kPer = 8;
        const int g_e = e / group_experts;  // device of this expert
        uint32_t info[kPer], rank[kPer];
        bool c[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int tl = tid + NT * j;
            const int t = b * seg_tokens + tl;
            info[j] = tl < seg_tokens ? key_s[pad(tl)] : 0u;
            c[j] = tl < seg_tokens && ((info[j] >> 20) != 0u || (EXPANDED && t / group_tokens == g_e));
            // rank within the class, below 2^30: score bits (scores are in [0,1]), position, or a draw
            rank[j] = 0u;
            if (c[j]) {
                if (metric == MOE_METRIC_ORDER)
                    rank[j] = (uint32_t)(seg_tokens - 1 - tl);
                else if (metric == MOE_METRIC_REVERSE_ORDER)
                    rank[j] = (uint32_t)tl;
                else if (metric == MOE_METRIC_RANDOM)
                    rank[j] = pair_hash(seed, (uint32_t)t * (uint32_t)E + (uint32_t)e) >> 3;
                else
                    rank[j] = __float_as_uint(scores[(size_t)t * E + e]);
                if (token_class) rank[j] += (uint32_t)(token_class[t] & 3) << 30;
            }
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int tl = tid + NT * j;
            if (tl >= seg_tokens) continue;
            const int t = b * seg_tokens + tl;
            int below = (int)(info[j] & 1023u);
            const int listed = (int)((info[j] >> 10) & 1023u);
            if (EXPANDED) {
                const int lower = e - (t / group_tokens) * group_experts;  // experts of the token's device below e
                below += lower < 0 ? 0 : (lower > group_experts ? group_experts : lower);
            }
            const uint32_t key = c[j] ? rank[j] + 1u : 0u;
            if (c[j]) atomicAdd(&hist[key >> 24], 1);
            key_s[pad(tl)] = key;
            slot_s[tl] = (uint8_t)below;
            if (e == 0) {  // slots beyond the token's candidate count stay unused
                const int n_c = listed + (EXPANDED ? group_experts : 0);
                for (int sl = n_c; sl < S; ++sl) pair_row[(size_t)t * S + sl] = -1;
            }
        }
    }
    __syncthreads();

    // ---- kept rows of every segment: this block's first row, its expert's total ----
    int before = 0, own_total = 0, n_cand = 0;
    for (int i = tid; i < segs; i += NT) {
        int c = 0;
        for (int r = 0; r < copies; ++r) c += cand[r * pitch + i];
        const int bb = i / E, ee = i - bb * E;
        if (EXPANDED) {  // plus the tokens of block bb that sit on the expert's device
            const int lo = (ee / group_experts) * group_tokens, hi = lo + group_tokens;
            const int s0 = bb * seg_tokens, s1 = s0 + seg_tokens;
            const int a = lo > s0 ? lo : s0, z = hi < s1 ? hi : s1;
            c += z > a ? z - a : 0;
        }
        const int kept = c < cap ? c : cap;
        if (scheduler) atomicAdd(&sched_tot[ee], kept);
        if (ee < e || (ee == e && bb < b)) before += kept;
        if (ee == e) own_total += kept;
        if (i == seg) n_cand = c;
    }
    // block sums of the three (one pair of barriers)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        before += __shfl_xor(before, off, kWave);
        own_total += __shfl_xor(own_total, off, kWave);
        n_cand += __shfl_xor(n_cand, off, kWave);
    }
    if (lane == 0) {
        red3[wv][0] = before;
        red3[wv][1] = own_total;
        red3[wv][2] = n_cand;
    }
    __syncthreads();
    int row0 = 0, total;
    own_total = n_cand = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        row0 += red3[w][0];
        own_total += red3[w][1];
        n_cand += red3[w][2];
    }
    if (tid == 0) {
        seg_count[seg] = n_cand < cap ? n_cand : cap;
        if (b == 0) {
            expert_count[e] = own_total;
            expert_offset[e] = row0;
            if (e == E - 1) expert_offset[E] = row0 + own_total;
        }
    }

    // ---- threshold: keys above tau are kept, `need` of the keys equal to tau are kept (Eq. 8) ----
    uint32_t tau = 0;  // every candidate (key >= 1) passes
    int need = 0;
    if (cap == 0) {
        tau = 0xffffffffu;  // nothing passes
    } else if (n_cand > cap) {
        // cap-th largest key, most significant byte first; the histogram of the top byte is already there
        uint32_t prefix = 0;
        need = cap;
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (shift != 24) {
                __syncthreads();
                if (tid < 256) hist[tid] = 0;
                __syncthreads();
                const uint32_t hi_mask = 0xffffffffu << (shift + 8);
                for (int tl = tid; tl < seg_tokens; tl += NT) {
                    const uint32_t kx = key_s[pad(tl)];
                    if (kx != 0u && (kx & hi_mask) == prefix) atomicAdd(&hist[(kx >> shift) & 255u], 1);
                }
                __syncthreads();
            }
            // the first wave owns the digits, lane l the four digits 255-4l .. 252-4l: a scan over its lanes
            // counts the keys with a larger digit; the digit where that count first reaches `need` holds the
            // cap-th key
            if (wv == 0) {
                int h[4], sum = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    h[u] = hist[255 - 4 * lane - u];
                    sum += h[u];
                }
                int incl = sum;
#pragma unroll
                for (int off = 1; off < kWave; off <<= 1) {
                    const int o = __shfl_up(incl, off, kWave);
                    if (lane >= off) incl += o;
                }
                int above = incl - sum;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (above < need && above + h[u] >= need) {  // exactly one lane and digit
                        sh_prefix = prefix | ((uint32_t)(255 - 4 * lane - u) << shift);
                        sh_rem = need - above;
                    }
                    above += h[u];
                }
            }
            __syncthreads();
            prefix = sh_prefix;
            need = sh_rem;
        }
        tau = prefix;
    }

    // ---- ordered compaction: rows in ascending token order, ties at the threshold to the lower tokens ----
    const int run = (seg_tokens + NT - 1) / NT;  // at most 8
    const int tb = tid * run;
    uint32_t kx[8];
    int eq_cnt = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        kx[j] = j < run && tb + j < seg_tokens ? key_s[pad(tb + j)] : 0u;
        eq_cnt += kx[j] != 0u && kx[j] == tau;
    }
    int eq_rank = fused_exclusive_scan<NT>(eq_cnt, red, &total);
    uint32_t keep_bits = 0;
    int keep_cnt = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bool c = kx[j] != 0u;
        const bool eq = c && kx[j] == tau;
        const bool keep = c && (kx[j] > tau || (eq && eq_rank < need));
        eq_rank += eq;
        keep_cnt += keep;
        keep_bits |= (uint32_t)keep << j;
    }
    int pos = row0 + fused_exclusive_scan<NT>(keep_cnt, red, &total);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (kx[j] == 0u) continue;
        const int t = b * seg_tokens + tb + j;
        const bool keep = (keep_bits >> j) & 1u;
        if (keep) {
            row_token[pos] = t;
            // the gating score, whatever ranked the pair (under the Score metric it is the key itself)
            row_weight[pos] = weight_from_key ? __uint_as_float(kx[j] - 1u) : scores[(size_t)t * E + e];
        }
        pair_row[(size_t)t * S + slot_s[tb + j]] = keep ? pos : -1;
        pos += keep;
    }
    if (scheduler) {
        __syncthreads();
        build_schedule_from_totals(sched_tot, sched_off, sched);
    }
}

hipError_t launch_capacity_drop(const moe_desc_t& d, const Sizes& s, const DropWorkspace& ws, const float* scores,
                                const int32_t* topk_idx, const uint8_t* token_class, uint32_t seed,
                                int32_t* expert_count, int32_t* seg_count,
                                int32_t* expert_offset, int32_t* row_token, float* row_weight, int32_t* pair_row,
                                const FfnScheduleArgs* schedule, hipStream_t st) {
    const int N = d.n_tokens, E = d.n_experts;
    FfnScheduleArgs no_schedule = {};  // enabled = 0
    const FfnScheduleArgs& sched = schedule ? *schedule : no_schedule;
    {
        const int segs_all = s.n_blocks * E;
        constexpr int kSmallBlock = 256;  // threads of a block for short segments of short batches
        const bool fused = s.span == 1 && !(d.max_experts && s.slots > d.top_k) && N > 0 &&
                           s.seg_tokens <= kFusedMaxTokens && segs_all + 1 <= kFusedCounters &&
                           segs_all <= kFusedMaxSegs && (long long)segs_all * N * s.list_k <= kFusedMaxWork;
        if (fused) {
            // every block reads all N lists: small blocks only where that is a single round for them too
            const bool small = s.seg_tokens <= 8 * kSmallBlock && N <= 8 * kSmallBlock;
            const bool ex = d.mode == MOE_MODE_EXPANDED_DROP, one = s.n_blocks == 1;
            auto launch = [&](auto kern, int threads) {
                ProfileScope prof(MOE_KERNEL_DROP_SELECT, st);
                hipLaunchKernelGGL(kern, dim3(segs_all), dim3(threads), 0, st, scores, topk_idx, token_class, seed,
                                   expert_count, seg_count, expert_offset, row_token, row_weight, pair_row, N, E, s.list_k,
                                   s.slots, s.group_tokens, s.group_experts, d.metric, s.seg_tokens, s.n_blocks, s.cap,
                                   d.metric == MOE_METRIC_SCORE && !token_class ? 1 : 0, sched);
            };
            auto by_size = [&](auto ex_c, auto one_c, auto vw_c) {
                constexpr bool EX = decltype(ex_c)::value, ONE = decltype(one_c)::value;
                constexpr int VW = decltype(vw_c)::value;
                if (small)
                    launch(drop_fused_kernel<EX, ONE, VW, kSmallBlock>, kSmallBlock);
                else
                    launch(drop_fused_kernel<EX, ONE, VW, kFusedThreads>, kFusedThreads);
            };
            auto by_width = [&](auto ex_c, auto one_c) {
                if (s.list_k % 4 == 0)
                    by_size(ex_c, one_c, std::integral_constant<int, 4>{});
                else if (s.list_k % 2 == 0)
                    by_size(ex_c, one_c, std::integral_constant<int, 2>{});
                else
                    by_size(ex_c, one_c, std::integral_constant<int, 1>{});
            };
            if (ex && one)
                by_width(std::true_type{}, std::true_type{});
            else if (ex)
                by_width(std::true_type{}, std::false_type{});
            else if (one)
                by_width(std::false_type{}, std::true_type{});
            else
                by_width(std::false_type{}, std::false_type{});
            return hipGetLastError();
        }
    }
    if (N > 0) {
        const int grid = (N + kPrepTokens - 1) / kPrepTokens;
        const size_t lds = (size_t)kPrepTokens * (E | 1) * 5;
        if (lds > 64 * 1024)
            (void)hipFuncSetAttribute((const void*)drop_prepare_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)lds);
        ProfileScope prof(MOE_KERNEL_DROP_PREPARE, st);
        hipLaunchKernelGGL(drop_prepare_kernel, dim3(grid), dim3(256), lds, st, scores, topk_idx, ws.key_t, ws.slot_t,
                           pair_row, N, E, s.list_k, s.slots, d.mode == MOE_MODE_EXPANDED_DROP ? 1 : 0, s.group_tokens,
                           s.group_experts, d.metric, s.seg_tokens > 0 ? s.seg_tokens : 1, token_class, seed);
    }
    const int segs = s.n_blocks * E;
    {
        ProfileScope prof(MOE_KERNEL_DROP_SELECT, st);
        const size_t n_keys = (size_t)s.seg_tokens * s.span;
        const size_t lds = (n_keys <= (size_t)kSelectCache ? n_keys : 0) * 4;
        static std::atomic<uint64_t> configured{0};
        once_per_device(configured, [] {  // up to 128 KB of keys plus the kernel's own few kilobytes
            for (const void* k : {(const void*)drop_select_kernel<256, 1>, (const void*)drop_select_kernel<256, 4>,
                                  (const void*)drop_select_kernel<1024, 1>, (const void*)drop_select_kernel<1024, 4>})
                (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kSelectCache * 4);
        });
        const bool wide = n_keys > 4096;                          // threads per block
        const bool vec = N % 4 == 0 && s.seg_tokens % 4 == 0;     // 16-byte loads of four keys
        auto kern = wide ? (vec ? drop_select_kernel<1024, 4> : drop_select_kernel<1024, 1>)
                         : (vec ? drop_select_kernel<256, 4> : drop_select_kernel<256, 1>);
        hipLaunchKernelGGL(kern, dim3(segs / s.span), dim3(wide ? 1024 : 256), lds, st, ws.key_t, ws.seg_tau,
                           ws.seg_need, seg_count, N, E, s.seg_tokens, s.span, s.cap);
    }
    auto emit = [&](bool last) {
        ProfileScope prof(MOE_KERNEL_DROP_EMIT, st);
        const int parts = s.seg_tokens > kEmitChunk ? (s.seg_tokens + kEmitChunk - 1) / kEmitChunk : 1;
        hipLaunchKernelGGL(drop_emit_kernel, dim3(segs * parts), dim3(256), 0, st, scores, ws.key_t, ws.slot_t, ws.seg_tau,
                           ws.seg_need, seg_count, expert_count, expert_offset, row_token, row_weight, pair_row, N, E,
                           s.n_blocks, s.seg_tokens, s.slots, d.metric == MOE_METRIC_SCORE && !token_class ? 1 : 0,
                           last ? sched : no_schedule);
    };
    const bool limit = d.max_experts && s.slots > d.top_k && N > 0;
    emit(!limit);
    if (limit) {
        // the first plan tells which pairs survive the capacity; trim every token to k of them, emit again
        // the key tile of 64 tokens and their rows of pair_row: at most 256 * 65 + 64 * 255 words
        const size_t lds = ((size_t)E * kLimitPitch + (size_t)kLimitTokens * s.slots) * 4;
        auto kern = E <= 64 ? drop_limit_kernel<1> : (E <= 128 ? drop_limit_kernel<2> : drop_limit_kernel<4>);
        if (lds > 48 * 1024)
            (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        {
            ProfileScope prof(MOE_KERNEL_DROP_LIMIT, st);
            hipLaunchKernelGGL(kern, dim3((N + kLimitTokens - 1) / kLimitTokens), dim3(256), lds, st, scores, ws.key_t,
                               pair_row, ws.seg_tau, ws.seg_need, seg_count, N, E, s.slots, d.top_k, s.seg_tokens, segs);
        }
        emit(true);
    }
    return hipGetLastError();
}

}  // namespace capmoe
