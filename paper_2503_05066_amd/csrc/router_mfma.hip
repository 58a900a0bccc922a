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

#include <type_traits>

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

// two fp32 router weights -> one word of each bf16 plane (w = hi + mid + lo exactly)
__device__ inline void split_pair(float v0, float v1, uint32_t& h, uint32_t& m, uint32_t& l) {
    // the bf16 of the first element is the word's low half, of the second one its high half
    h = bf16_pair(v0, v1);
    const float r0 = v0 - __uint_as_float(h << 16);
    const float r1 = v1 - __uint_as_float(h & 0xffff0000u);
    m = bf16_pair(r0, r1);
    const float q0 = r0 - __uint_as_float(m << 16);
    const float q1 = r1 - __uint_as_float(m & 0xffff0000u);
    l = bf16_pair(q0, q1);
}

template <int N, class F, int I = 0>
__device__ inline void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, F, I + 1>(static_cast<F&&>(f));
    }
}

// LDS bytes of one stage: three planes of 32*TN rows of 32 bf16, plus (when the planes' 16-byte
// pieces do not divide among 256 threads) 2 KB where the threads without a piece put their stores
constexpr int rm_stage_bytes(int tn) { return 3 * 32 * tn * 64 + ((32 * tn * 4) % 256 != 0 ? 2048 : 0); }

// TN = 32-expert tiles of a block (blockIdx.z picks the block's 32*TN experts; the last block's are padded).  out: [ksplit, N, E] partial sums (or the logits
// themselves, with the bias added, when there is a single slice).
// D = depth of the register ring of requested slabs; it divides the slabs of a slice.
template <int TN, int D>
__global__ __launch_bounds__(256) void router_mfma_kernel(const uint16_t* __restrict__ x, const float* __restrict__ w,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int N, int d, int E, int k_per_slice, int add_bias) {
    constexpr int EP = 32 * TN;                  // padded expert count
    constexpr int PLANE = EP * 64;               // EP rows of 32 bf16 (64 bytes)
    constexpr int STAGE_BYTES = rm_stage_bytes(TN);
    constexpr int NP = (EP * 4 + 255) / 256;     // 16-byte pieces of a plane that a thread stages
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int lr = lane & 31, lk = lane >> 5;
    const int t0 = blockIdx.x * kRmTokens + wv * 32;
    const int slice = blockIdx.y;
    const int e0 = blockIdx.z * EP;               // this block's experts: [e0, e0 + El)
    const int El = E - e0 < EP ? E - e0 : EP;
    const int k_begin = slice * k_per_slice;
    const int n_slabs = k_per_slice / kRmSlab;

    // this lane's token row (clamped: rows past N repeat the last token and are not stored)
    const int tr = t0 + lr < N ? t0 + lr : N - 1;
    const uint16_t* xrow = x + (size_t)tr * d + k_begin + lk * 8;

    // weight pieces this thread stages: piece p = row p/4 (expert), 8 consecutive k at (p%4)*8.
    // Padding rows repeat the last expert; a thread whose last piece lies past the planes (odd TN)
    // still loads and splits it, and stores it to the spare 2 KB of the stage: no branches in the loop.
    const float* wsrc[NP];
    int wdst[NP][3];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int p = tid + 256 * i;
        const int e = p >> 2, kc = p & 3;
        wsrc[i] = w + (size_t)(e0 + (e < El ? e : El - 1)) * d + k_begin + kc * 8;
        const int at = e * 64 + ((kc ^ ((e >> 2) & 3)) << 4);  // EP is a multiple of 4: same swizzle per plane
#pragma unroll
        for (int q = 0; q < 3; ++q) wdst[i][q] = p < EP * 4 ? q * PLANE + at : 3 * PLANE + (tid & 127) * 16;
    }
    // Register ring of D slabs: the fp32 weights and the token fragments of slab s + D are requested
    // while slab s is multiplied, so that a block keeps D slabs of loads in flight.  The loop below
    // has no branches: the compiler's wait counts are exact only when every path issues the same
    // loads (with a request under a condition it waited for nearly all of them, which emptied the
    // ring), so a request past the slice is made all the same, from one fixed address.
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
            w_off[p][i] = p * PLANE + R * 64 + ((lk ^ ((R >> 2) & 3)) << 4);
        }

    // slab s -> ring slot; past the slice: values nobody uses, all lanes on one cache line
    auto request_w = [&](auto slot, int s) {
        constexpr int u = decltype(slot)::value;
        const bool live = s < n_slabs;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const float* src = live ? wsrc[i] + s * kRmSlab : w;
            wreg[u][i][0] = *(const float4*)src;
            wreg[u][i][1] = *(const float4*)(src + 4);
        }
    };
    auto request_x = [&](auto slot, int s) {
        constexpr int u = decltype(slot)::value;
        const uint16_t* xs = s < n_slabs ? xrow + s * kRmSlab : x;
        xreg[u][0] = *(const bf16x8*)xs;
        xreg[u][1] = *(const bf16x8*)(xs + 16);
    };

    // One slab: 6*TN MFMAs on the planes in stage `st` (per k-step the smallest plane first, consecutive
    // MFMAs to different accumulators), their operand reads issued PD fragments ahead; the
    // weights in ring slot `un` are split and stored to stage `nx` between the MFMAs, a pair of weights
    // at a time, so that the vector unit works under the matrix unit.  The scheduling barriers keep
    // the compiler from regrouping the steps (it otherwise reads two fragments, waits, multiplies).
    constexpr int F = 6 * TN, PD = F < 8 ? F : 8, NC = NP * 4;
    auto slab = [&](auto slot_next, const uint8_t* st, uint8_t* nx, const bf16x8& xa0, const bf16x8& xa1) {
        constexpr int un = decltype(slot_next)::value;
        bf16x8 wf[F];
        uint32_t h[NP][4], m[NP][4], l[NP][4];
        auto read = [&](auto fc) {
            constexpr int f = decltype(fc)::value;
            constexpr int ks = f / (3 * TN), p = 2 - (f / TN) % 3, i = f % TN;
            wf[f] = *(const bf16x8*)(st + (w_off[p][i] ^ (ks << 5)));
        };
        static_for<PD>(read);
        static_for<F>([&](auto fc) {
            constexpr int f = decltype(fc)::value;
            constexpr int ks = f / (3 * TN), i = f % TN;
            if constexpr (f + PD < F) read(std::integral_constant<int, f + PD>{});
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[f], ks == 0 ? xa0 : xa1, acc[i], 0, 0, 0);
            static_for<NC>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                if constexpr (c * F / NC == f) {
                    constexpr int pc = c / 4, j = c % 4;
                    const float4 v = wreg[un][pc][j / 2];
                    if constexpr (j % 2 == 0) split_pair(v.x, v.y, h[pc][j], m[pc][j], l[pc][j]);
                    else split_pair(v.z, v.w, h[pc][j], m[pc][j], l[pc][j]);
                    if constexpr (j == 3) {
                        *(uint4*)(nx + wdst[pc][0]) = make_uint4(h[pc][0], h[pc][1], h[pc][2], h[pc][3]);
                        *(uint4*)(nx + wdst[pc][1]) = make_uint4(m[pc][0], m[pc][1], m[pc][2], m[pc][3]);
                        *(uint4*)(nx + wdst[pc][2]) = make_uint4(l[pc][0], l[pc][1], l[pc][2], l[pc][3]);
                    }
                }
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    static_for<D>([&](auto c) {
        request_w(c, decltype(c)::value);
        request_x(c, decltype(c)::value);
    });
    // slab 0 goes to stage 0 before the loop
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        uint32_t h[4], m[4], l[4];
        split_pair(wreg[0][i][0].x, wreg[0][i][0].y, h[0], m[0], l[0]);
        split_pair(wreg[0][i][0].z, wreg[0][i][0].w, h[1], m[1], l[1]);
        split_pair(wreg[0][i][1].x, wreg[0][i][1].y, h[2], m[2], l[2]);
        split_pair(wreg[0][i][1].z, wreg[0][i][1].w, h[3], m[3], l[3]);
        *(uint4*)(smem + wdst[i][0]) = make_uint4(h[0], h[1], h[2], h[3]);
        *(uint4*)(smem + wdst[i][1]) = make_uint4(m[0], m[1], m[2], m[3]);
        *(uint4*)(smem + wdst[i][2]) = make_uint4(l[0], l[1], l[2], l[3]);
    }
    request_w(std::integral_constant<int, 0>{}, D);
    // One barrier per slab: the stage written during slab s was last read during slab s - 1, which
    // every wave has left when it arrives at the barrier of slab s.  During the last slab the stage
    // that nobody reads again receives the split of a request past the slice.
    for (int s0 = 0; s0 < n_slabs; s0 += D) {
        static_for<D>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int un = (u + 1) % D;
            const int sl = s0 + u;
            const uint8_t* st = smem + (sl & 1) * STAGE_BYTES;
            uint8_t* nx = smem + ((sl + 1) & 1) * STAGE_BYTES;
            __syncthreads();
            // slab sl is multiplied while the weights of slab sl + 1 are split; both ring slots are
            // free after that (each slot is requested again only when its old value is dead, so the
            // ring stays in fixed registers)
            slab(std::integral_constant<int, un>{}, st, nx, xreg[u][0], xreg[u][1]);
            request_w(std::integral_constant<int, un>{}, sl + 1 + D);
            request_x(uc, sl + D);
        });
    }

    // lane holds token (lane & 31) and experts 8q + 4*(lane/32) + v of each 32-expert tile: four
    // consecutive experts go out as one 16-byte store where the row allows it (4-byte stores cost a
    // quarter of the kernel; passing whole rows through LDS gains nothing more)
    const int t = t0 + lr;
    if (t < N) {
        float* orow = out + ((size_t)slice * N + t) * E + e0;
        const bool vec = (E & 3) == 0;  // rows stay 16-byte aligned
        const bool biased = add_bias && bias != nullptr;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = i * 32 + q * 8 + lk * 4;
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    // clamped index: the loads do not depend on one another or on a branch per element
                    const float b = biased ? bias[e0 + (e + v < El ? e + v : El - 1)] : 0.f;
                    o[v] = acc[i][q * 4 + v] + b;
                }
                if (vec && e + 3 < El) {
                    *(float4*)(orow + e) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (e + v < El) orow[e + v] = o[v];
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
    const int tiles = (d.n_experts + 31) / 32;
    const int blocks_m = (d.n_tokens + kRmTokens - 1) / kRmTokens * (tiles >= 4 ? 2 : 1);
    int want = (256 + blocks_m - 1) / blocks_m;  // aim at one block per compute unit or more
    if (want > 32) want = 32;
    // the largest count of slices up to that whose slices are whole slabs, with a multiple of four
    // slabs each if there is such a count (the kernel's ring of requests is then four deep)
    int ks = 1, ks4 = 0;
    for (int c = 1; c <= want; ++c) {
        if (d.d_model % (c * kRmSlab) == 0) ks = c;
        if (d.d_model % (c * kRmSlab * 4) == 0) ks4 = c;
    }
    w.ksplit = ks4 > 0 ? ks4 : ks;
    char* p = (char*)base;
    size_t off = 0;
    if (ks > 1) {
        w.partial = (float*)(p + off);
        off += align256((size_t)ks * d.n_tokens * d.n_experts * 4);
    }
    w.bytes = off;
    return w;
}

template <int TN, int D>
static void launch_rm_depth(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w,
                            const float* bias, float* out, hipStream_t st) {
    const size_t lds = (size_t)2 * rm_stage_bytes(TN);
    auto kern = router_mfma_kernel<TN, D>;
    static std::atomic<uint64_t> configured{0};
    once_per_device(configured, [&] {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    const dim3 grid((d.n_tokens + kRmTokens - 1) / kRmTokens, ws.ksplit, (d.n_experts + 32 * TN - 1) / (32 * TN));
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const uint16_t*)x, w, bias, out, d.n_tokens, d.d_model,
                       d.n_experts, d.d_model / ws.ksplit, ws.ksplit == 1 ? 1 : 0);
}

// the deepest ring (up to 4 slabs) that divides the slabs of a slice
template <int TN>
static void launch_rm(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w, const float* bias,
                      float* out, hipStream_t st) {
    const int n_slabs = d.d_model / ws.ksplit / kRmSlab;
    if (n_slabs % 4 == 0) return launch_rm_depth<TN, 4>(d, ws, x, w, bias, out, st);
    if (n_slabs % 2 == 0) return launch_rm_depth<TN, 2>(d, ws, x, w, bias, out, st);
    launch_rm_depth<TN, 1>(d, ws, x, w, bias, out, st);
}

// Writes either the logits (single K slice) or ws.partial (several slices, summed later).
hipError_t launch_router_mfma(const moe_desc_t& d, const RouteWorkspace& ws, const void* x, const float* w,
                              const float* bias, float* logits, hipStream_t st) {
    ProfileScope prof(MOE_KERNEL_ROUTER_LOGITS, st);
    float* out = ws.ksplit == 1 ? logits : ws.partial;
    // From 97 experts up two blocks share a token tile, each with half of the 32-expert tiles: two
    // blocks per compute unit hide more than x fetched a second time (from L2) costs (128 experts,
    // 16 384 tokens: 39 -> 37 us; splitting 64 experts the same way is slower, 10.8 -> 11.9 us).
    const int tiles = (d.n_experts + 31) / 32;
    switch (tiles >= 4 ? (tiles + 1) / 2 : tiles) {
        case 1: launch_rm<1>(d, ws, x, w, bias, out, st); break;
        case 2: launch_rm<2>(d, ws, x, w, bias, out, st); break;
        case 3: launch_rm<3>(d, ws, x, w, bias, out, st); break;
        default: launch_rm<4>(d, ws, x, w, bias, out, st); break;
    }
    return hipGetLastError();
}

}  // namespace capmoe
