// Router: logits = x W_r^T + b, softmax over experts and top-k (Eq. 1).
//
// This translation unit is compiled with -ffp-contract=off: the softmax is a fixed sequence of
// individually rounded fp32 operations, so equal logits give bit-equal scores on any conforming
// implementation of the same sequence.
#include <hip/hip_bf16.h>

#include "common.h"

namespace capmoe {

// ---------------------------------------------------------------------------------------------
// Router logits: a skinny GEMM [N,d] x [d,E], fp32 accumulation.
// One block computes 64 tokens x all experts; K is walked in slabs of 32 staged in LDS.
// Thread (ty,tx) of a 16x16 block owns tokens ty*4..+3 and experts tx + 16*i.
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ inline float load_as_float(const T* p);
template <>
__device__ inline float load_as_float<float>(const float* p) {
    return *p;
}
template <>
__device__ inline float load_as_float<__hip_bfloat16>(const __hip_bfloat16* p) {
    return __uint_as_float((uint32_t)(*(const uint16_t*)p) << 16);
}

constexpr int kRtTokens = 64;
constexpr int kRtSlab = 32;

template <typename T, int EPT>
__global__ __launch_bounds__(256) void router_logits_kernel(const T* __restrict__ x, const float* __restrict__ w,
                                                            const float* __restrict__ bias,
                                                            float* __restrict__ logits, int N, int d, int E) {
    extern __shared__ float smem[];
    float* xs = smem;                               // [64][33]
    float* wsm = smem + kRtTokens * (kRtSlab + 1);  // [16*EPT][33]
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int t0 = blockIdx.x * kRtTokens;
    const int e_rows = 16 * EPT;

    float acc[4][EPT];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < EPT; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < d; k0 += kRtSlab) {
        for (int idx = tid; idx < kRtTokens * kRtSlab; idx += 256) {
            const int r = idx >> 5, c = idx & 31;
            const int t = t0 + r, kk = k0 + c;
            xs[r * (kRtSlab + 1) + c] = (t < N && kk < d) ? load_as_float<T>(x + (size_t)t * d + kk) : 0.f;
        }
        for (int idx = tid; idx < e_rows * kRtSlab; idx += 256) {
            const int r = idx >> 5, c = idx & 31;
            const int kk = k0 + c;
            wsm[r * (kRtSlab + 1) + c] = (r < E && kk < d) ? w[(size_t)r * d + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < kRtSlab; ++c) {
            float xv[4], wv[EPT];
#pragma unroll
            for (int i = 0; i < 4; ++i) xv[i] = xs[(ty * 4 + i) * (kRtSlab + 1) + c];
#pragma unroll
            for (int j = 0; j < EPT; ++j) wv[j] = wsm[(tx + 16 * j) * (kRtSlab + 1) + c];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < EPT; ++j) acc[i][j] = __builtin_fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty * 4 + i;
        if (t >= N) continue;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int e = tx + 16 * j;
            if (e < E) logits[(size_t)t * E + e] = acc[i][j] + (bias ? bias[e] : 0.f);
        }
    }
}

template <typename T, int EPT>
static void launch_rl(const T* x, const float* w, const float* bias, float* logits, int N, int d, int E,
                      hipStream_t st) {
    const int grid = (N + kRtTokens - 1) / kRtTokens;
    const size_t lds = sizeof(float) * (kRtSlab + 1) * (kRtTokens + 16 * EPT);
    hipLaunchKernelGGL((router_logits_kernel<T, EPT>), dim3(grid), dim3(256), lds, st, x, w, bias, logits, N, d, E);
}

template <typename T>
static void dispatch_rl(const T* x, const float* w, const float* bias, float* logits, int N, int d, int E,
                        hipStream_t st) {
    const int ept = (E + 15) / 16;
    if (ept <= 1)
        launch_rl<T, 1>(x, w, bias, logits, N, d, E, st);
    else if (ept <= 2)
        launch_rl<T, 2>(x, w, bias, logits, N, d, E, st);
    else if (ept <= 4)
        launch_rl<T, 4>(x, w, bias, logits, N, d, E, st);
    else if (ept <= 8)
        launch_rl<T, 8>(x, w, bias, logits, N, d, E, st);
    else if (ept <= 16)
        launch_rl<T, 16>(x, w, bias, logits, N, d, E, st);
    else
        launch_rl<T, 32>(x, w, bias, logits, N, d, E, st);
}

hipError_t launch_router_logits(const moe_desc_t& d, const void* x, const float* w, const float* bias, float* logits,
                                hipStream_t st) {
    ProfileScope prof(MOE_KERNEL_ROUTER_LOGITS, st);
    if (d.dtype == MOE_DTYPE_BF16)
        dispatch_rl<__hip_bfloat16>((const __hip_bfloat16*)x, w, bias, logits, d.n_tokens, d.d_model, d.n_experts, st);
    else
        dispatch_rl<float>((const float*)x, w, bias, logits, d.n_tokens, d.d_model, d.n_experts, st);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Softmax + top-k, one wavefront per token; lane l owns experts l, l+64, ...
//
// exp(z), z <= 0, by a fixed fp32 sequence: cut to zero below -80 (keeps every later value a
// normal number), n = rint(z*log2 e), r = z - n*ln2 in two fused steps, degree-7 Taylor polynomial
// by Horner with fused multiply-adds, scaling by 2^n.  The denominator is the sum of the
// numerators in ascending expert order; the quotient is an IEEE division.
// ---------------------------------------------------------------------------------------------
__device__ inline float exp_nonpositive(float z) {
    if (z < -80.0f) return 0.0f;
    const float n = __builtin_rintf(__fmul_rn(z, 0x1.715476p+0f));
    float r = __builtin_fmaf(n, -0x1.62e400p-1f, z);
    r = __builtin_fmaf(n, -0x1.7f7d1cp-20f, r);
    float q = 0x1.a01a02p-13f;
    q = __builtin_fmaf(q, r, 0x1.6c16c2p-10f);
    q = __builtin_fmaf(q, r, 0x1.111112p-7f);
    q = __builtin_fmaf(q, r, 0x1.555556p-5f);
    q = __builtin_fmaf(q, r, 0x1.555556p-3f);
    q = __builtin_fmaf(q, r, 0.5f);
    q = __builtin_fmaf(q, r, 1.0f);
    q = __builtin_fmaf(q, r, 1.0f);
    return __builtin_ldexpf(q, (int)n);
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

template <int EPL>
__global__ __launch_bounds__(256) void softmax_topk_kernel(float* __restrict__ logits,
                                                           const float* __restrict__ partial, int ksplit,
                                                           const float* __restrict__ bias, float* __restrict__ scores,
                                                           int32_t* __restrict__ topk_idx,
                                                           float* __restrict__ topk_score, int N, int E, int k) {
    __shared__ __attribute__((aligned(16))) float numer[4][EPL * kWave];
    __shared__ uint2 winners[4][kMaxTopK];  // (score bits, expert) of a token's k winners, ascending expert
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    // a wave works alone: its LDS row is private, and LDS operations of one wave complete in order
    for (int base = blockIdx.x * 4; base < N; base += gridDim.x * 4) {
        const int t = base + wv;
        const bool live = t < N;
        if (!live) break;
        float* l = logits + (size_t)(live ? t : 0) * E;
        float v[EPL];
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + kWave * i;
            if (e < E && partial) {
                // the router GEMM left one partial sum per K slice: add them in slice order
                // (eight loads in flight at a time: one dependent load per addition costs a microsecond each)
                float sum = bias ? bias[e] : 0.0f;
                for (int s0 = 0; s0 < ksplit; s0 += 8) {
                    float p[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        p[u] = s0 + u < ksplit ? partial[((size_t)(s0 + u) * N + t) * E + e] : 0.0f;
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (s0 + u < ksplit) sum = __fadd_rn(sum, p[u]);
                }
                v[i] = sum;
                if (live) l[e] = sum;
            } else {
                v[i] = e < E ? l[e] : -INFINITY;
            }
            m = fmaxf(m, v[i]);
        }
        m = wave_max(m);
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + kWave * i;
            v[i] = e < E ? exp_nonpositive(__fsub_rn(v[i], m)) : 0.0f;
            numer[wv][e] = v[i];
        }
        __builtin_amdgcn_wave_barrier();
        // every lane adds the numerators in ascending expert order (same address for all lanes, four per
        // read; the entries past E are +0 and leave the sum as it is)
        float sum = 0.0f;
        for (int e = 0; e < E; e += 4) {
            const float4 n4 = *(const float4*)&numer[wv][e];
            sum = __fadd_rn(__fadd_rn(__fadd_rn(__fadd_rn(sum, n4.x), n4.y), n4.z), n4.w);
        }
        __builtin_amdgcn_wave_barrier();  // the row is rewritten for the wave's next token only after these reads
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + kWave * i;
            v[i] = __fdiv_rn(v[i], sum);
            if (e < E)
                scores[(size_t)t * E + e] = v[i];
            else
                v[i] = -1.0f;
        }
        // top-k by selection: scores are >= +0, so their bit patterns order like the values.
        // (1) the k-th largest pattern by a 30-step binary search on ballots (1.0f has bit 29 as its highest),
        // (2) winners = patterns above it, plus the lowest expert ids among those equal to it,
        // (3) every winner finds its place (larger score first, then lower expert id) by counting the
        //     winners ahead of it in a list the wave keeps in LDS.
        // Repeated wave-wide arg-max costs k rounds of cross-lane steps; this is a few ballots per bit.
        uint32_t bits[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) bits[i] = __float_as_uint(v[i] < 0.0f ? 0.0f : v[i]);
        uint32_t tau = 0;
        for (int bit = 29; bit >= 0; --bit) {
            const uint32_t cand = tau | (1u << bit);
            int cnt = 0;
#pragma unroll
            for (int i = 0; i < EPL; ++i) cnt += __popcll(__ballot(lane + kWave * i < E && bits[i] >= cand));
            if (cnt >= k) tau = cand;
        }
        int n_gt = 0;
#pragma unroll
        for (int i = 0; i < EPL; ++i) n_gt += __popcll(__ballot(lane + kWave * i < E && bits[i] > tau));
        const int need = k - n_gt;  // >= 1: how many of the patterns equal to tau win
        const uint64_t below = (1ull << lane) - 1ull;
        int eq_before = 0, win_before = 0;
        uint2* list = &winners[wv][0];
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int e = lane + kWave * i;
            const bool valid = e < E;
            const bool eq = valid && bits[i] == tau;
            const uint64_t eq_mask = __ballot(eq);
            const bool win = valid && (bits[i] > tau || (eq && eq_before + __popcll(eq_mask & below) < need));
            const uint64_t win_mask = __ballot(win);
            if (win) list[win_before + __popcll(win_mask & below)] = make_uint2(bits[i], (uint32_t)e);
            eq_before += __popcll(eq_mask);
            win_before += __popcll(win_mask);
            if (!win) bits[i] = 0xffffffffu;  // marks "no output"
        }
        __builtin_amdgcn_wave_barrier();
        int place[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) place[i] = 0;
        for (int j = 0; j < k; ++j) {
            const uint2 w = list[j];  // same address in every lane
#pragma unroll
            for (int i = 0; i < EPL; ++i)
                place[i] += (w.x > bits[i] || (w.x == bits[i] && (int)w.y < lane + kWave * i)) ? 1 : 0;
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i)
            if (bits[i] != 0xffffffffu) {
                topk_idx[(size_t)t * k + place[i]] = lane + kWave * i;
                topk_score[(size_t)t * k + place[i]] = __uint_as_float(bits[i]);
            }
        __builtin_amdgcn_wave_barrier();  // the list is rewritten for the wave's next token only after these reads
    }
}

hipError_t launch_softmax_topk(const moe_desc_t& d, float* logits, const float* partial, int ksplit, const float* bias,
                               float* scores, int32_t* topk_idx, float* topk_score, hipStream_t st) {
    ProfileScope prof(MOE_KERNEL_SOFTMAX_TOPK, st);
    const int N = d.n_tokens, E = d.n_experts, k = d.top_k + d.overselect;
    int grid = (N + 3) / 4;
    if (grid > 2048) grid = 2048;
    const int epl = (E + kWave - 1) / kWave;
    if (epl <= 1)
        hipLaunchKernelGGL((softmax_topk_kernel<1>), dim3(grid), dim3(256), 0, st, logits, partial, ksplit, bias, scores,
                           topk_idx, topk_score, N, E, k);
    else if (epl <= 2)
        hipLaunchKernelGGL((softmax_topk_kernel<2>), dim3(grid), dim3(256), 0, st, logits, partial, ksplit, bias, scores,
                           topk_idx, topk_score, N, E, k);
    else if (epl <= 4)
        hipLaunchKernelGGL((softmax_topk_kernel<4>), dim3(grid), dim3(256), 0, st, logits, partial, ksplit, bias, scores,
                           topk_idx, topk_score, N, E, k);
    else
        hipLaunchKernelGGL((softmax_topk_kernel<8>), dim3(grid), dim3(256), 0, st, logits, partial, ksplit, bias, scores,
                           topk_idx, topk_score, N, E, k);
    return hipGetLastError();
}

}  // namespace capmoe
