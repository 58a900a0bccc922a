// Expert computation E_i(x) of Eq. (2): a grouped SwiGLU FFN over the expert-major rows.
//
//   hidden[r,:] = silu(W_gate[e] xp[r,:]) * (W_up[e] xp[r,:])        (GEMM 1, fused epilogue)
//   yp[r,:]     = W_down[e] hidden[r,:]                               (GEMM 2)
//
// Rows per expert are only known on the device, so a one-block kernel first turns expert_offset
// into a list of row tiles (expert, first row, valid rows); the GEMM grids are sized for the
// static upper bound and surplus blocks exit at once.
//
// bf16: both operands are K-contiguous ("NT" GEMM), staged through LDS in 16-byte pieces with an
// XOR swizzle, multiplied on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
// The weight rows feed the MFMA's first operand and the activation rows the second, so a lane
// ends up with 4 consecutive output columns of one row and stores them as one 8-byte piece.
#include "common.h"

namespace capmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// ---------------------------------------------------------------------------------------------
// tile schedule
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void ffn_schedule_kernel(const int32_t* __restrict__ expert_offset, int E, int tile_m,
                                                          int32_t* __restrict__ tile_expert,
                                                          int32_t* __restrict__ tile_row0,
                                                          int32_t* __restrict__ tile_rows,
                                                          int32_t* __restrict__ n_tiles, int max_tiles) {
    const int lane = threadIdx.x;
    int base = 0;
    for (int e0 = 0; e0 < E; e0 += kWave) {
        const int e = e0 + lane;
        const int lo = e < E ? expert_offset[e] : 0;
        const int hi = e < E ? expert_offset[e + 1] : 0;
        const int nt = (hi - lo + tile_m - 1) / tile_m;
        int incl = nt;  // inclusive scan over the wave
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const int o = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += o;
        }
        const int first = base + incl - nt;
        for (int i = 0; i < nt; ++i) {
            const int idx = first + i;
            if (idx < max_tiles) {
                tile_expert[idx] = e;
                tile_row0[idx] = lo + i * tile_m;
                const int left = hi - (lo + i * tile_m);
                tile_rows[idx] = left < tile_m ? left : tile_m;
            }
        }
        base += __shfl(incl, kWave - 1, kWave);
    }
    if (lane == 0) *n_tiles = base < max_tiles ? base : max_tiles;
}

// ---------------------------------------------------------------------------------------------
// fp32 path (small layers): one 16x16 output tile per block, K walked in slabs of 16.
// ---------------------------------------------------------------------------------------------
template <bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(const float* __restrict__ A,
                                                               const float* __restrict__ B0,
                                                               const float* __restrict__ B1, float* __restrict__ C,
                                                               const int32_t* __restrict__ tile_expert,
                                                               const int32_t* __restrict__ tile_row0,
                                                               const int32_t* __restrict__ tile_rows,
                                                               const int32_t* __restrict__ n_tiles, int K, int Nout) {
    __shared__ float as[16][17], b0s[16][17], b1s[16][17];
    const int nt = *n_tiles;
    if (nt == 0) return;
    const int tile = blockIdx.x % nt, nb = blockIdx.x / nt;  // row tiles vary fastest
    if (nb * 16 >= Nout) return;
    const int e = tile_expert[tile], row0 = tile_row0[tile], rows = tile_rows[tile];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n0 = nb * 16;
    const float* b0 = B0 + (size_t)e * Nout * K;
    const float* b1 = SWIGLU ? B1 + (size_t)e * Nout * K : nullptr;
    float acc0 = 0.f, acc1 = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
        const int kk = k0 + tx;
        as[ty][tx] = (ty < rows && kk < K) ? A[(size_t)(row0 + ty) * K + kk] : 0.f;
        b0s[ty][tx] = (n0 + ty < Nout && kk < K) ? b0[(size_t)(n0 + ty) * K + kk] : 0.f;
        if (SWIGLU) b1s[ty][tx] = (n0 + ty < Nout && kk < K) ? b1[(size_t)(n0 + ty) * K + kk] : 0.f;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            acc0 = fmaf(as[ty][c], b0s[tx][c], acc0);
            if (SWIGLU) acc1 = fmaf(as[ty][c], b1s[tx][c], acc1);
        }
        __syncthreads();
    }
    if (ty < rows && n0 + tx < Nout) {
        float out = acc0;
        if (SWIGLU) out = acc0 / (1.0f + expf(-acc0)) * acc1;
        C[(size_t)(row0 + ty) * Nout + n0 + tx] = out;
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA path
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    const uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    const uint32_t ra = (a + 0x7fffu + ((a >> 16) & 1u)) >> 16;
    const uint32_t rb = (b + 0x7fffu + ((b >> 16) & 1u)) & 0xffff0000u;
    return ra | rb;
}

// Block tile: BM activation rows x BN weight rows, K slab BK; 4 waves as 2 (M) x 2 (N).
// SWIGLU: weight rows [0,BN/2) of the tile come from W_gate, [BN/2,BN) from W_up, for the same
// BN/2 hidden columns; a wave holds matching gate and up columns and applies silu(g)*u itself.
template <int BM, int BN, int BK, bool SWIGLU>
__global__ __launch_bounds__(256) void grouped_gemm_bf16_kernel(const uint16_t* __restrict__ A,
                                                                const uint16_t* __restrict__ B0,
                                                                const uint16_t* __restrict__ B1,
                                                                uint16_t* __restrict__ C,
                                                                const int32_t* __restrict__ tile_expert,
                                                                const int32_t* __restrict__ tile_row0,
                                                                const int32_t* __restrict__ tile_rows,
                                                                const int32_t* __restrict__ n_tiles, int K, int Nout) {
    constexpr int CPR = BK / 8;             // 16-byte pieces per tile row
    constexpr int WM = BM / 2, WN = BN / 2;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PIECES = BM * CPR / 256, B_PIECES = BN * CPR / 256;
    constexpr int STAGE = (BM + BN) * BK;  // bf16 elements per stage
    static_assert(CPR == 8 || CPR == 4, "BK must be 32 or 64");
    static_assert(BM % 64 == 0 && BN % 64 == 0, "tile shape");
    static_assert(!SWIGLU || TN % 2 == 0, "a wave needs matching gate and up columns");

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    const int ncols = SWIGLU ? BN / 2 : BN;  // output columns per block
    const int nt = *n_tiles;
    if (nt == 0) return;
    const int tile = blockIdx.x % nt, nb = blockIdx.x / nt;  // row tiles vary fastest
    if (nb * ncols >= Nout) return;
    const int e = tile_expert[tile], row0 = tile_row0[tile], rows = tile_rows[tile];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv & 1, wn = wv >> 1;
    const int n0 = nb * ncols;

    // per-thread source pointers of the pieces this thread stages
    const uint16_t* a_src[A_PIECES];
    const uint16_t* b_src[B_PIECES];
    int a_dst[A_PIECES], b_dst[B_PIECES];
#pragma unroll
    for (int i = 0; i < A_PIECES; ++i) {
        const int c = tid + 256 * i, r = c / CPR, kc = c % CPR;
        const int rr = r < rows ? r : rows - 1;  // rows past the expert's end repeat its last row
        a_src[i] = A + (size_t)(row0 + rr) * K + kc * 8;
        a_dst[i] = (r * CPR + (kc ^ (CPR == 8 ? (r & 7) : ((r >> 1) & 3)))) * 8;
    }
#pragma unroll
    for (int i = 0; i < B_PIECES; ++i) {
        const int c = tid + 256 * i, r = c / CPR, kc = c % CPR;
        const uint16_t* base;
        if (SWIGLU)
            base = (r < BN / 2 ? B0 + ((size_t)e * Nout + n0 + r) * K : B1 + ((size_t)e * Nout + n0 + r - BN / 2) * K);
        else
            base = B0 + ((size_t)e * Nout + n0 + r) * K;
        b_src[i] = base + kc * 8;
        b_dst[i] = BM * BK + (r * CPR + (kc ^ (CPR == 8 ? (r & 7) : ((r >> 1) & 3)))) * 8;
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 a_reg[A_PIECES], b_reg[B_PIECES];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_PIECES; ++i) a_reg[i] = *(const uint4*)(a_src[i] + (size_t)kt * BK);
#pragma unroll
        for (int i = 0; i < B_PIECES; ++i) b_reg[i] = *(const uint4*)(b_src[i] + (size_t)kt * BK);
    };
    auto store_lds = [&](int buf) {
        uint16_t* s = smem + buf * STAGE;
#pragma unroll
        for (int i = 0; i < A_PIECES; ++i) *(uint4*)(s + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_PIECES; ++i) *(uint4*)(s + b_dst[i]) = b_reg[i];
    };

    // LDS row of the weight sub-tile tn of this wave (SWIGLU: first half gate, second half up)
    auto w_row = [&](int tn) {
        if (SWIGLU) {
            const int half = tn / (TN / 2), idx = tn % (TN / 2);
            return half * (BN / 2) + wn * (WN / 2) + idx * 32;
        }
        return wn * WN + tn * 32;
    };

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int lr = lane & 31, lk = lane >> 5;
    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_global(kt + 1);
        const uint16_t* s = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kc = ks * 2 + lk;
            bf16x8 xa[TM], wb[TN];
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int r = wm * WM + j * 32 + lr;
                xa[j] = *(const bf16x8*)(s + (r * CPR + (kc ^ (CPR == 8 ? (r & 7) : ((r >> 1) & 3)))) * 8);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const int r = w_row(i) + lr;
                wb[i] = *(const bf16x8*)(s + BM * BK + (r * CPR + (kc ^ (CPR == 8 ? (r & 7) : ((r >> 1) & 3)))) * 8);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[i], xa[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: lane holds, for activation row (lane & 31) of each 32-row sub-tile, output columns
    // 8*(v/4) + 4*(lane/32) + (v%4) of each 32-column sub-tile
    constexpr int TNO = SWIGLU ? TN / 2 : TN;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = wm * WM + j * 32 + lr;
        if (r >= rows) continue;
        uint16_t* crow = C + (size_t)(row0 + r) * Nout + n0;
#pragma unroll
        for (int i = 0; i < TNO; ++i) {
            const int cbase = (SWIGLU ? wn * (WN / 2) : wn * WN) + i * 32 + 4 * lk;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float o[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float g = acc[i][j][q * 4 + v];
                    if (SWIGLU) {
                        const float u = acc[i + TN / 2][j][q * 4 + v];
                        o[v] = g / (1.0f + __expf(-g)) * u;
                    } else {
                        o[v] = g;
                    }
                }
                uint2 pk;
                pk.x = pack_bf16x2(o[0], o[1]);
                pk.y = pack_bf16x2(o[2], o[3]);
                *(uint2*)(crow + cbase + q * 8) = pk;
            }
        }
    }
}

template <int BM, int BN, int BK, bool SWIGLU>
static void launch_bf16(const void* A, const void* B0, const void* B1, void* C, const FfnWorkspace& ws, int K, int Nout,
                        hipStream_t st) {
    ProfileScope prof(SWIGLU ? MOE_KERNEL_FFN_GATE_UP : MOE_KERNEL_FFN_DOWN, st);
    const int ncols = SWIGLU ? BN / 2 : BN;
    const size_t lds = (size_t)2 * (BM + BN) * BK * 2;
    auto kern = grouped_gemm_bf16_kernel<BM, BN, BK, SWIGLU>;
    static bool configured = false;
    if (!configured) {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((Nout / ncols) * ws.max_tiles), dim3(256), lds, st, (const uint16_t*)A,
                       (const uint16_t*)B0, (const uint16_t*)B1, (uint16_t*)C, ws.tile_expert, ws.tile_row0,
                       ws.tile_rows, ws.n_tiles, K, Nout);
}

hipError_t launch_grouped_ffn(const moe_desc_t& d, const Sizes& s, const FfnWorkspace& ws, const void* xp,
                              const int32_t* expert_offset, const void* w_gate, const void* w_up, const void* w_down,
                              void* yp, hipStream_t st) {
    (void)s;
    {
        ProfileScope prof(MOE_KERNEL_FFN_SCHEDULE, st);
        hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(64), 0, st, expert_offset, d.n_experts, ws.tile_m,
                           ws.tile_expert, ws.tile_row0, ws.tile_rows, ws.n_tiles, ws.max_tiles);
    }
    if (d.dtype == MOE_DTYPE_BF16) {
        launch_bf16<kFfnTileM, 128, 64, true>(xp, w_gate, w_up, ws.hidden, ws, d.d_model, d.d_hidden, st);
        launch_bf16<kFfnTileM, 128, 64, false>(ws.hidden, w_down, nullptr, yp, ws, d.d_hidden, d.d_model, st);
    } else {
        const dim3 g1(((d.d_hidden + 15) / 16) * ws.max_tiles), g2(((d.d_model + 15) / 16) * ws.max_tiles);
        {
            ProfileScope prof(MOE_KERNEL_FFN_GATE_UP, st);
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<true>), g1, dim3(256), 0, st, (const float*)xp,
                           (const float*)w_gate, (const float*)w_up, (float*)ws.hidden, ws.tile_expert, ws.tile_row0,
                           ws.tile_rows, ws.n_tiles, d.d_model, d.d_hidden);
        }
        ProfileScope prof(MOE_KERNEL_FFN_DOWN, st);
        hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), g2, dim3(256), 0, st, (const float*)ws.hidden,
                           (const float*)w_down, (const float*)nullptr, (float*)yp, ws.tile_expert, ws.tile_row0,
                           ws.tile_rows, ws.n_tiles, d.d_hidden, d.d_model);
    }
    return hipGetLastError();
}

}  // namespace capmoe
