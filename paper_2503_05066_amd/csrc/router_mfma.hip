// Router logits for bf16 activations on the matrix cores, at fp32 accuracy.
//
// The router weight is fp32.  It is split exactly into three bf16 planes, w = hi + mid + lo
// (8 + 8 + 8 significand bits); x is bf16 already, so every product x*plane is exact in fp32 and
// the three MFMAs of a k-step accumulate into one fp32 accumulator: the result is an fp32-accurate
// dot product computed at bf16 matrix rate (3 MFMAs instead of one fp32-rate GEMM).
//
// Work split: a block owns 128 tokens (4 waves x 32) and one slice of K; the slices' partial sums
// are added, in slice order, by the softmax kernel (deterministic: no floating-point atomics).
// The fp32 weights of a 32-wide k-slab are split in registers and the three planes go to LDS
// (shared by the 4 waves, two stages); each wave reads its own 32 token rows straight from global
// memory.  Loads run several slabs ahead of the multiplication in a register ring.
#include "common.h"

namespace capmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

constexpr int kRmTokens = 128;  // tokens per block
constexpr int kRmSlab = 32;     // k per LDS stage

// two floats -> two bf16 (round to nearest even) in one word, the first in the low half: the hardware conversion
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ inline uint32_t bf16_pair(float a, float b) {
    const f32x2_t v = {a, b};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return *(const uint32_t*)&r;
}

// 8 fp32 router weights -> the three bf16 planes (w = hi + mid + lo exactly), 16 bytes each
__device__ inline void split_planes(const float4& a, const float4& b, uint4& hi, uint4& mid, uint4& lo) {
    const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // a pair at a time; the bf16 of the even element is the word's low half, of the odd one its high half
        h[i] = bf16_pair(v[2 * i], v[2 * i + 1]);
        const float r0 = v[2 * i] - __uint_as_float(h[i] << 16);
        const float r1 = v[2 * i + 1] - __uint_as_float(h[i] & 0xffff0000u);
        m[i] = bf16_pair(r0, r1);
        const float q0 = r0 - __uint_as_float(m[i] << 16);
        const float q1 = r1 - __uint_as_float(m[i] & 0xffff0000u);
        l[i] = bf16_pair(q0, q1);
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    mid = make_uint4(m[0], m[1], m[2], m[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// TN = 32-expert tiles (E padded to 32*TN).  out: [ksplit, N, E] partial sums (or the logits
// themselves, with the bias added, when there is a single slice).
template <int TN>
__global__ __launch_bounds__(256) void router_mfma_kernel(const uint16_t* __restrict__ x, const float* __restrict__ w,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int N, int d, int E, int k_per_slice, int add_bias) {
    constexpr int EP = 32 * TN;                  // padded expert count
    constexpr int STAGE_BYTES = 3 * EP * 64;     // three planes of EP rows, 32 bf16 (64 bytes) each
    constexpr int NP = (EP * 4 + 255) / 256;     // 16-byte pieces of a plane that a thread stages
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int lr = lane & 31, lk = lane >> 5;
    const int t0 = blockIdx.x * kRmTokens + wv * 32;
    const int slice = blockIdx.y;
    const int k_begin = slice * k_per_slice;
    const int n_slabs = k_per_slice / kRmSlab;

    // this lane's token row (clamped: rows past N repeat the last token and are not stored)
    const int tr = t0 + lr < N ? t0 + lr : N - 1;
    const uint16_t* xrow = x + (size_t)tr * d + k_begin + lk * 8;

    // weight pieces this thread stages: piece p = row p/4 (expert), 8 consecutive k at (p%4)*8
    const float* wsrc[NP];
    int wdst[NP];
    bool wlive[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int p = tid + 256 * i;
        const int e = p >> 2, kc = p & 3;
        wlive[i] = p < EP * 4;
        wsrc[i] = w + (size_t)(e < E ? e : E - 1) * d + k_begin + kc * 8;  // padding rows repeat the last expert
        wdst[i] = e * 64 + ((kc ^ ((e >> 2) & 3)) << 4);                   // EP is a multiple of 4: same swizzle per plane
    }
    // Register ring of D slabs: the fp32 weights and the token fragments of slab s + D are requested
    // while slab s is multiplied, so that a block keeps D slabs of loads in flight (the kernel is
    // bound by load latency: a slab is only 6 * TN MFMAs of work per wave).
    constexpr int D = TN <= 4 ? 4 : 2;
    float4 wreg[D][NP][2];
    bf16x8 xreg[D][2];

    f32x16 acc[TN];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // LDS offsets of this lane's weight pieces for k-step 0 (piece lk); k-step 1 flips piece bit 1
    int w_off[3][TN];
#pragma unroll
    for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int R = i * 32 + lr;
            w_off[p][i] = p * EP * 64 + R * 64 + ((lk ^ ((R >> 2) & 3)) << 4);
        }

#pragma unroll
    for (int u = 0; u < D; ++u) {
        if (u < n_slabs) {
#pragma unroll
            for (int i = 0; i < NP; ++i)
                if (wlive[i]) {
                    wreg[u][i][0] = *(const float4*)(wsrc[i] + u * kRmSlab);
                    wreg[u][i][1] = *(const float4*)(wsrc[i] + u * kRmSlab + 4);
                }
            xreg[u][0] = *(const bf16x8*)(xrow + u * kRmSlab);
            xreg[u][1] = *(const bf16x8*)(xrow + u * kRmSlab + 16);
        }
    }
    for (int s0 = 0; s0 < n_slabs; s0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int sl = s0 + u;
            if (sl < n_slabs) {  // block-uniform
                uint8_t* st = smem + (sl & 1) * STAGE_BYTES;
                // split this slab's weights into the three planes of the stage the previous slab does not use
#pragma unroll
                for (int i = 0; i < NP; ++i)
                    if (wlive[i]) {
                        uint4 hi, mid, lo;
                        split_planes(wreg[u][i][0], wreg[u][i][1], hi, mid, lo);
                        *(uint4*)(st + wdst[i]) = hi;
                        *(uint4*)(st + EP * 64 + wdst[i]) = mid;
                        *(uint4*)(st + 2 * EP * 64 + wdst[i]) = lo;
                    }
                const bf16x8 xa0 = xreg[u][0], xa1 = xreg[u][1];
                if (sl + D < n_slabs) {  // refill the slot
#pragma unroll
                    for (int i = 0; i < NP; ++i)
                        if (wlive[i]) {
                            wreg[u][i][0] = *(const float4*)(wsrc[i] + (sl + D) * kRmSlab);
                            wreg[u][i][1] = *(const float4*)(wsrc[i] + (sl + D) * kRmSlab + 4);
                        }
                    xreg[u][0] = *(const bf16x8*)(xrow + (sl + D) * kRmSlab);
                    xreg[u][1] = *(const bf16x8*)(xrow + (sl + D) * kRmSlab + 16);
                }
                // one barrier per slab: the stage written now was last read two slabs ago, i.e. before
                // the previous barrier
                __syncthreads();
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                    for (int i = 0; i < TN; ++i) {
                        // smallest plane first
#pragma unroll
                        for (int p = 2; p >= 0; --p) {
                            const bf16x8 wf = *(const bf16x8*)(st + (w_off[p][i] ^ (ks << 5)));
                            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, ks == 0 ? xa0 : xa1, acc[i], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // lane holds token (lane & 31) and experts 8q + 4*(lane/32) + v of each 32-expert tile: four
    // consecutive experts go out as one 16-byte store where the row allows it (4-byte stores cost a
    // quarter of the kernel; passing whole rows through LDS gains nothing more)
    const int t = t0 + lr;
    if (t < N) {
        float* orow = out + ((size_t)slice * N + t) * E;
        const bool vec = (E & 3) == 0;  // rows stay 16-byte aligned
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = i * 32 + q * 8 + lk * 4;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    o[v] = acc[i][q * 4 + v] + (add_bias && bias && e + v < E ? bias[e + v] : 0.f);
                if (vec && e + 3 < E) {
                    *(float4*)(orow + e) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (e + v < E) orow[e + v] = o[v];
                }
            }
    }
}

RouteWorkspace route_workspace(const moe_desc_t& d, void* base) {
    RouteWorkspace w;
    w.use_mfma = d.dtype == MOE_DTYPE_BF16 && d.d_model % 32 == 0 && d.n_tokens > 0;
    w.ksplit = 1;
    w.partial = nullptr;
    w.bytes = 0;
    if (!w.use_mfma) return w;
    const int blocks_m = (d.n_tokens + kRmTokens - 1) / kRmTokens;
    int want = (256 + blocks_m - 1) / blocks_m;  // aim at one block per compute unit or more
    if (want > 32) want = 32;
    int ks = 1;
    for (int c = 1; c <= want; ++c)
        if (d.d_model % (c * kRmSlab) == 0) ks = c;
    w.ksplit = ks;
    char* p = (char*)base;
    size_t off = 0;
    if (ks > 1) {
        w.partial = (float*)(p + off);
        off += align256((size_t)ks * d.n_tokens * d.n_experts * 4);
    }
    w.bytes = off;
    return w;
}

template <int TN>
static void launch_rm(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w, const float* bias,
                      float* out, hipStream_t st) {
    (void)ws;
    const size_t lds = (size_t)2 * 3 * 32 * TN * 64;
    auto kern = router_mfma_kernel<TN>;
    static bool configured = false;
    if (!configured) {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    const dim3 grid((d.n_tokens + kRmTokens - 1) / kRmTokens, ws.ksplit);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const uint16_t*)x, w, bias, out, d.n_tokens, d.d_model,
                       d.n_experts, d.d_model / ws.ksplit, ws.ksplit == 1 ? 1 : 0);
}

// Writes either the logits (single K slice) or ws.partial (several slices, summed later).
hipError_t launch_router_mfma(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w,
                              const float* bias, float* logits, hipStream_t st) {
    ProfileScope prof(MOE_KERNEL_ROUTER_LOGITS, st);
    float* out = ws.ksplit == 1 ? logits : ws.partial;
    const int tn = (d.n_experts + 31) / 32;
    switch (tn) {
        case 1: launch_rm<1>(d, ws, x, w, bias, out, st); break;
        case 2: launch_rm<2>(d, ws, x, w, bias, out, st); break;
        case 3: launch_rm<3>(d, ws, x, w, bias, out, st); break;
        case 4: launch_rm<4>(d, ws, x, w, bias, out, st); break;
        case 5: launch_rm<5>(d, ws, x, w, bias, out, st); break;
        case 6: launch_rm<6>(d, ws, x, w, bias, out, st); break;
        case 7: launch_rm<7>(d, ws, x, w, bias, out, st); break;
        default: launch_rm<8>(d, ws, x, w, bias, out, st); break;
    }
    return hipGetLastError();
}

}  // namespace capmoe
