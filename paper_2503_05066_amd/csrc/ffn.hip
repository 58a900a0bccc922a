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

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Block tile: BM activation rows x BN weight rows, K slab of 64; WAVES_M x WAVES_N wavefronts.
//
// LDS holds two stages; a stage is (BM + BN) rows of 128 bytes.  Rows are filled by direct
// global->LDS loads: one wave-wide load writes 8 rows (64 lanes x 16 bytes, contiguous in LDS), and
// each lane chooses WHICH 16-byte piece of its row it fetches, so that piece kc of row r lands at
// position kc ^ ((r >> 1) & 7): with 64 LDS banks a 16-lane group of a 16-byte read then touches
// 16 different bank groups, for the fill as well as for the MFMA operand reads.
//
// SWIGLU: weight rows [0,BN/2) of the tile come from W_gate, [BN/2,BN) from W_up, for the same
// BN/2 hidden columns; a wave holds matching gate and up columns and applies silu(g)*u itself.
//
// Blocks are numbered so that each XCD (block id mod 8) walks a contiguous range of tiles, ordered
// [column group][row tile][column in group]: blocks that run together share row and weight tiles in
// their XCD's L2.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWIGLU>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void ffn_gemm_bf16_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1,
    uint16_t* __restrict__ C, const int32_t* __restrict__ tile_expert, const int32_t* __restrict__ tile_row0,
    const int32_t* __restrict__ tile_rows, const int32_t* __restrict__ n_tiles, int K, int Nout, int col_group) {
    constexpr int BK = 64;
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int A_GROUPS = BM / 8, GROUPS = (BM + BN) / 8;  // 8-row groups of a stage
    constexpr int LOADS = GROUPS / NW;                         // wave-wide loads per wave per stage
    constexpr int STAGE_BYTES = (BM + BN) * 128;
    constexpr int NCOLS = SWIGLU ? BN / 2 : BN;  // output columns per block
    static_assert(GROUPS % NW == 0, "loads must divide evenly over the waves");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile");
    static_assert(!SWIGLU || TN % 2 == 0, "a wave needs matching gate and up columns");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    // ---- which tile ----
    const int nt = *n_tiles;
    const int nb_total = Nout / NCOLS;
    const int total = nt * nb_total;
    const int chunk = (total + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int logical = xcd * chunk + slot;
    if (slot >= chunk || logical >= total) return;
    const int per_group = nt * col_group;
    const int cg = logical / per_group, rem = logical - cg * per_group;
    const int tile = rem / col_group, nb = cg * col_group + (rem - tile * col_group);
    const int e = tile_expert[tile], row0 = tile_row0[tile], rows = tile_rows[tile];
    const int n0 = nb * NCOLS;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WAVES_M, wn = wv / WAVES_M;

    // ---- sources of this lane's pieces ----
    const uint16_t* src[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int g = wv + NW * i;           // row group inside the stage (wave-uniform)
        const int r = g * 8 + (lane >> 3);   // row inside the stage: A rows first, then weight rows
        const int kc = (lane & 7) ^ ((r >> 1) & 7);
        if (g < A_GROUPS) {
            const int rr = r < rows ? r : rows - 1;  // rows past the expert's end repeat its last row
            src[i] = A + (size_t)(row0 + rr) * K + kc * 8;
        } else {
            const int rb = r - BM;
            if (SWIGLU && rb >= BN / 2)
                src[i] = B1 + ((size_t)e * Nout + n0 + rb - BN / 2) * K + kc * 8;
            else
                src[i] = B0 + ((size_t)e * Nout + n0 + rb) * K + kc * 8;
        }
    }

    // ---- LDS offsets of this lane's operand pieces (k-step 0; later steps flip piece bits) ----
    const int lr = lane & 31, lk = lane >> 5;
    int a_off[TM], a_sw[TM], b_off[TN], b_sw[TN];
    bool m_live[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = wm * WTM + j * 32 + lr;
        a_off[j] = r * 128;
        a_sw[j] = (r >> 1) & 7;
        m_live[j] = wm * WTM + j * 32 < rows;  // wave-uniform: skip sub-tiles past the expert's end
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
        int r;
        if (SWIGLU) {
            const int half = i / (TN / 2), idx = i % (TN / 2);
            r = half * (BN / 2) + wn * (WTN / 2) + idx * 32 + lr;
        } else {
            r = wn * WTN + i * 32 + lr;
        }
        b_off[i] = BM * 128 + r * 128;
        b_sw[i] = (r >> 1) & 7;
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int KT = K / BK;
    // prologue: stage 0
#pragma unroll
    for (int i = 0; i < LOADS; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)src[i], (lptr_t)(smem + (wv + NW * i) * 1024), 16, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's pieces have landed
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) {
            uint8_t* dst = smem + (cur ^ 1) * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < LOADS; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t)(src[i] + (size_t)(kt + 1) * BK),
                                                 (lptr_t)(dst + (wv + NW * i) * 1024), 16, 0, 0);
        }
        const uint8_t* s = smem + cur * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int kc = ks * 2 + lk;
            bf16x8 xa[TM], wb[TN];
#pragma unroll
            for (int j = 0; j < TM; ++j)
                if (m_live[j]) xa[j] = *(const bf16x8*)(s + a_off[j] + ((kc ^ a_sw[j]) << 4));
#pragma unroll
            for (int i = 0; i < TN; ++i) wb[i] = *(const bf16x8*)(s + b_off[i] + ((kc ^ b_sw[i]) << 4));
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    if (m_live[j]) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[i], xa[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
    }

    // ---- epilogue: a lane holds, for activation row (lane & 31) of each 32-row sub-tile, output
    // columns 8*q + 4*(lane/32) + v (q, v = 0..3) of each 32-column sub-tile ----
    constexpr int TNO = SWIGLU ? TN / 2 : TN;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = wm * WTM + j * 32 + lr;
        if (r >= rows) continue;
        uint16_t* crow = C + (size_t)(row0 + r) * Nout + n0;
#pragma unroll
        for (int i = 0; i < TNO; ++i) {
            const int cbase = (SWIGLU ? wn * (WTN / 2) : wn * WTN) + i * 32 + 4 * lk;
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

static int column_group(int nb_total) {
    for (int g = 4; g > 1; --g)
        if (nb_total % g == 0) return g;
    return 1;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWIGLU>
static void launch_bf16(const void* A, const void* B0, const void* B1, void* C, const FfnWorkspace& ws, int K, int Nout,
                        hipStream_t st) {
    ProfileScope prof(SWIGLU ? MOE_KERNEL_FFN_GATE_UP : MOE_KERNEL_FFN_DOWN, st);
    constexpr int NCOLS = SWIGLU ? BN / 2 : BN;
    const size_t lds = (size_t)2 * (BM + BN) * 128;
    auto kern = ffn_gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, SWIGLU>;
    static bool configured = false;
    if (!configured) {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    const int nb_total = Nout / NCOLS;
    const long long grid = (long long)nb_total * ws.max_tiles + 8;  // + 8: every XCD gets a whole chunk
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(64 * WAVES_M * WAVES_N), lds, st, (const uint16_t*)A,
                       (const uint16_t*)B0, (const uint16_t*)B1, (uint16_t*)C, ws.tile_expert, ws.tile_row0,
                       ws.tile_rows, ws.n_tiles, K, Nout, column_group(nb_total));
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
        launch_bf16<kFfnTileM, 256, 2, 4, true>(xp, w_gate, w_up, ws.hidden, ws, d.d_model, d.d_hidden, st);
        launch_bf16<kFfnTileM, 128, 2, 4, false>(ws.hidden, w_down, nullptr, yp, ws, d.d_hidden, d.d_model, st);
    } else {
        const dim3 g1(((d.d_hidden + 15) / 16) * ws.max_tiles), g2(((d.d_model + 15) / 16) * ws.max_tiles);
        {
            ProfileScope prof(MOE_KERNEL_FFN_GATE_UP, st);
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<true>), g1, dim3(256), 0, st, (const float*)xp,
                               (const float*)w_gate, (const float*)w_up, (float*)ws.hidden, ws.tile_expert,
                               ws.tile_row0, ws.tile_rows, ws.n_tiles, d.d_model, d.d_hidden);
        }
        ProfileScope prof(MOE_KERNEL_FFN_DOWN, st);
        hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), g2, dim3(256), 0, st, (const float*)ws.hidden,
                           (const float*)w_down, (const float*)nullptr, (float*)yp, ws.tile_expert, ws.tile_row0,
                           ws.tile_rows, ws.n_tiles, d.d_hidden, d.d_model);
    }
    return hipGetLastError();
}

}  // namespace capmoe
