// Expert computation E_i(x) of Eq. (2): a grouped SwiGLU FFN over the expert-major rows.
//
//   hidden[r,:] = silu(W_gate[e] xp[r,:]) * (W_up[e] xp[r,:])        (GEMM 1, fused epilogue)
//   yp[r,:]     = W_down[e] hidden[r,:]                               (GEMM 2)
//
// Rows per expert are only known on the device, so one wave (a kernel of its own, or the tail of the
// capacity drop's last launch) first turns expert_offset into lists of row tiles (expert, first row,
// valid rows); the GEMM grids are sized for the static upper bound and surplus blocks exit at once.
//
// bf16: both operands are K-contiguous ("NT" GEMM), staged through LDS in 16-byte pieces with an
// XOR swizzle and multiplied on the matrix cores with fp32 accumulation (v_mfma_f32_16x16x32_bf16 in
// both tile shapes): 256 x 256 blocks of 2 x 2 waves with 128 x 128 wave tiles for full-height row
// tiles (the bulk of the flops), 64 x 256 blocks of 1 x 4 waves with 64 x 64 wave tiles for the short
// remainders (weight streaming).  The weight rows feed the MFMA's first operand and the activation
// rows the second, so a lane ends up with 4 consecutive output columns of one row.
#include <type_traits>

#include "common.h"
#include "schedule.h"

namespace capmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

// ---------------------------------------------------------------------------------------------
// tile schedule (schedule.h) as a kernel of its own: one wave
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void ffn_schedule_kernel(const int32_t* __restrict__ expert_offset, FfnScheduleArgs args) {
    build_ffn_schedule(expert_offset, args);
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
                                                               const int32_t* __restrict__ n_tiles,
                                                               const int32_t* __restrict__ gather, int K, int Nout) {
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
    const int arow = ty < rows ? (gather ? gather[row0 + ty] : row0 + ty) : 0;
    for (int k0 = 0; k0 < K; k0 += 16) {
        const int kk = k0 + tx;
        as[ty][tx] = (ty < rows && kk < K) ? A[(size_t)arow * K + kk] : 0.f;
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
// two floats -> two bf16 (round to nearest even) in one word, lo in the low half: the hardware conversion
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *(const uint32_t*)&b;
}

typedef __attribute__((address_space(3))) void* lptr_t;

// s_waitcnt immediate for "at most n vector-memory operations outstanding, LDS/scalar counter
// at zero" (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at 7, lgkmcnt 11:8).
__host__ __device__ constexpr int waitcnt_vm(int n) { return (n & 15) | (7 << 4) | ((n >> 4) << 14); }

// What a wave needs to request its pieces of a K slab: one buffer descriptor per operand tensor (the
// block's activation rows, its weight rows, and for SwiGLU tiles the up-projection rows) and one 32-bit
// byte offset per wave-wide load.  Load i uses the activations for i < A_LOADS, the second weight tensor
// from B1_FROM on.  The loads are MUBUF loads with an LDS destination: unlike the global (FLAT-encoded)
// form, the compiler does not count them against the LDS counter, so the operand reads of the matrix
// loop keep fine-grained waits; the K advance goes into the scalar offset.
template <int LOADS, int A_LOADS, int B1_FROM>
struct Fills {
    static constexpr int kALoads = A_LOADS;
    __amdgpu_buffer_rsrc_t a, b0, b1;
    uint32_t voff[LOADS];
    __device__ __forceinline__ void one(int i, uint8_t* lds_dst, uint32_t k_bytes) const {
        // i is a compile-time constant after unrolling
        const __amdgpu_buffer_rsrc_t r = i < A_LOADS ? a : (i >= B1_FROM ? b1 : b0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lptr_t)lds_dst, 16, voff[i], k_bytes, 0, 0);
    }
};

// ---------------------------------------------------------------------------------------------
// tiles on 16x16x32 matrix instructions, four waves
// ---------------------------------------------------------------------------------------------
// Under sustained load the chip is power-limited, so what a kernel reaches is set by the energy it spends
// per flop.  Measured on this part with random operands: the 16x16x32 instruction sustains about 10 % more
// flops than 32x32x16 (half the accumulator traffic per flop), and a wave tile of 128 x 128 needs a third
// fewer LDS operand reads per flop than 128 x 64.  With one wave per SIMD nothing hides a stalled
// instruction, so the requests for the next slabs are spread over the whole slab (a burst of fills from
// every wave right after the barrier backs up the address unit and stalls the matrix pipe behind it).
typedef __attribute__((ext_vector_type(4))) float f32x4;

// c += a x b with the accumulator pinned to the accumulation registers: a wave of these tiles holds 256
// accumulator values, exactly the accumulation half of its register budget, and must never shuffle them
// through the other half.  The compiler does not see the instruction inside the statement, so the code
// that reads the accumulators after the last one waits out its latency itself.
__device__ __forceinline__ void mfma_16x16x32(f32x4& c, const bf16x8& a, const bf16x8& b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// K loop of a wave.  LDS: two slots of activation rows, then a ring of three slots of weight rows (the
// operand that streams from HBM gets a window of up to two slabs to land).  A slab is two 32-wide k-steps;
// matrix instructions lag the operand reads by one k-step:
//     k-step 0 of slab kt:  MFMAs  |  operand reads of k-step 1  |  requests for the weights of slab kt+2
//     barrier kt (slab kt+1 landed, slab kt no longer read)
//     k-step 1 of slab kt:  MFMAs  |  operand reads of slab kt+1 |  requests for the activations of slab kt+2
// Loads complete in order, so "all but the last B_LOADS" at barrier kt means the activations and weights of
// slab kt+1 have landed while the weights of slab kt+2 may still be in flight.  LIVE = number of 16-row
// activation sub-tiles that are multiplied (the rest lie past the expert's last row).
template <int BM, int BN, int NW, int TM, int TN, int WTN, bool SWIGLU, int LOADS, class FillsT>
struct PipelinedLoop16 {
    static constexpr int BK = 64;
    static constexpr int A_SLOT = BM * 128, B_SLOT = BN * 128, B_BASE = 2 * A_SLOT;
    static constexpr int LDS_BYTES = 2 * A_SLOT + 3 * B_SLOT;
    static constexpr int A_LOADS = FillsT::kALoads, B_LOADS = LOADS - A_LOADS;
    uint8_t* smem;
    const FillsT& fills;
    int a_lane, b_lane;  // byte offset, inside a slot, of this lane's piece of the wave's first row (k-step 0)
    int KT, wv;  // slabs this block multiplies, wave index
    int k0;      // first of them (0 unless the item is cut along K)

    // byte offset of weight sub-tile i relative to the wave's first weight row: with SwiGLU the second half
    // of the sub-tiles are the up-projection rows of the same hidden columns
    static __device__ __forceinline__ constexpr int b_tile(int i) {
        return SWIGLU ? ((i / (TN / 2)) * (BN / 2) + (i % (TN / 2)) * 16) * 128 : i * 16 * 128;
    }
    __device__ __forceinline__ uint32_t k_bytes(int kt) const { return (uint32_t)(kt + k0) * (BK * 2); }
    __device__ __forceinline__ void fill_a(int i, int kt) const {
        fills.one(i, smem + (kt & 1) * A_SLOT + (wv + NW * i) * 1024, k_bytes(kt));
    }
    __device__ __forceinline__ void fill_b(int i, int kt, int slot) const {
        fills.one(A_LOADS + i, smem + B_BASE + slot * B_SLOT + (wv + NW * i) * 1024, k_bytes(kt));
    }
    __device__ __forceinline__ void fill_a_all(int kt) const {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) fill_a(i, kt);
    }
    __device__ __forceinline__ void fill_b_all(int kt, int slot) const {
#pragma unroll
        for (int i = 0; i < B_LOADS; ++i) fill_b(i, kt, slot);
    }

    // PHASE (0..3): where in a k-step this wave places its fill requests.  The four waves leave every barrier
    // together and run the same instruction stream; with the same placement they would hand their requests to
    // the address unit in the same few cycles, its queue fills, and the waves that wait cannot issue their
    // next matrix instruction.  Each wave therefore shifts its requests by a different number of matrix
    // instructions.
    template <int LIVE, int PHASE = 0>
    __device__ __forceinline__ void run(f32x4 (&acc)[TN][TM]) const {
        fill_a_all(0);
        fill_b_all(0, 0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        __builtin_amdgcn_s_barrier();
        if (1 < KT) fill_a_all(1);
        if (1 < KT) fill_b_all(1, 1);
        if (LIVE == 0) {  // nothing to multiply in this wave: it only fills its share and keeps the barriers
            int slot2 = 2;  // slot of slab kt + 2
            for (int kt = 0; kt < KT; ++kt) {
                // as in the waves that multiply: the weights of slab kt+2 may still fly at the barrier
                if (kt + 2 < KT) {
                    fill_b_all(kt + 2, slot2);
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm(B_LOADS));
                } else {
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
                }
                __builtin_amdgcn_s_barrier();
                if (kt + 2 < KT) fill_a_all(kt + 2);
                slot2 = slot2 == 2 ? 0 : slot2 + 1;
            }
            return;
        }
        constexpr int NL = LIVE > 0 ? LIVE : 1;
        constexpr int NMFMA = TN * NL, NREAD = NL + TN;
        // reads go out in the first half of a k-step, so that they have returned long before the barrier
        constexpr int READ_EVERY = NMFMA / 2 / NREAD > 0 ? NMFMA / 2 / NREAD : 1;
        constexpr int B_EVERY = NMFMA / B_LOADS > 0 ? NMFMA / B_LOADS : 1;
        constexpr int A_EVERY = NMFMA / A_LOADS > 0 ? NMFMA / A_LOADS : 1;
        constexpr int B_OFF = PHASE * B_EVERY / 4 + (B_EVERY >= 8 ? B_EVERY / 8 : 0);
        constexpr int A_OFF = PHASE * A_EVERY / 4 + (A_EVERY >= 8 ? A_EVERY / 8 : 0);
        static_assert(B_OFF < B_EVERY && A_OFF < A_EVERY, "request placement");
        static_assert(LIVE == 0 || (NMFMA >= NREAD * READ_EVERY && NMFMA >= B_LOADS && NMFMA >= A_LOADS * A_EVERY), "k-step too short");
        bf16x8 xa[2][NL], wb[2][TN];

        // r-th operand read of a k-step, in the order the MFMAs (activation sub-tile major) need them:
        // weight 0, activation 0, weights 1.., activations 1..  pa / pb: this lane's piece of the wave's first
        // activation / weight row in the slot and k-step being read.
        auto read_item = [&](int r, int set, const uint8_t* pa, const uint8_t* pb) {
            if (r == 0)
                wb[set][0] = *(const bf16x8*)(pb + b_tile(0));
            else if (r == 1)
                xa[set][0] = *(const bf16x8*)(pa);
            else if (r <= TN)
                wb[set][r - 1] = *(const bf16x8*)(pb + b_tile(r - 1));
            else
                xa[set][r - TN] = *(const bf16x8*)(pa + (r - TN) * 16 * 128);
        };
#pragma unroll
        for (int r = 0; r < NREAD; ++r) read_item(r, 0, smem + a_lane, smem + B_BASE + b_lane);

        // One slab.  MORE: there is a next slab to read operands of; REFILL: slab kt+2 exists and is
        // requested.  Compile-time, so that the steady state carries no branches between its matrix
        // instructions; the last two slabs run the other instances.  slot = kt mod 3.
        auto slab = [&](int kt, int slot, auto more_c, auto refill_c) {
            constexpr bool MORE = decltype(more_c)::value, REFILL = decltype(refill_c)::value;
            const int slot2 = slot == 0 ? 2 : slot - 1;  // (kt + 2) mod 3
            const int next_slot = slot == 2 ? 0 : slot + 1;
            {
                // the second k-step's pieces sit four pieces further: bit 6 of the byte offset
                const uint8_t* pa = smem + (kt & 1) * A_SLOT + (a_lane ^ 64);
                const uint8_t* pb = smem + B_BASE + slot * B_SLOT + (b_lane ^ 64);
#pragma unroll
                for (int q = 0; q < NMFMA; ++q) {
                    const int j = q / TN, i = q % TN;
                    mfma_16x16x32(acc[i][j], wb[0][i], xa[0][j]);
                    if (q % READ_EVERY == 0 && q / READ_EVERY < NREAD) read_item(q / READ_EVERY, 1, pa, pb);
                    if (REFILL && q % B_EVERY == B_OFF && q / B_EVERY < B_LOADS) fill_b(q / B_EVERY, kt + 2, slot2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // slab kt+1 has landed for this wave (the younger weight requests may still fly), this wave's
            // operand reads of slab kt have returned (the LDS counter is part of the wait)
            if (REFILL)
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(B_LOADS));
            else
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            {
                const uint8_t* pa = smem + ((kt + 1) & 1) * A_SLOT + a_lane;
                const uint8_t* pb = smem + B_BASE + next_slot * B_SLOT + b_lane;
#pragma unroll
                for (int q = 0; q < NMFMA; ++q) {
                    const int j = q / TN, i = q % TN;
                    mfma_16x16x32(acc[i][j], wb[1][i], xa[1][j]);
                    if (MORE && q % READ_EVERY == 0 && q / READ_EVERY < NREAD) read_item(q / READ_EVERY, 0, pa, pb);
                    if (REFILL && q % A_EVERY == A_OFF && q / A_EVERY < A_LOADS) fill_a(q / A_EVERY, kt + 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        int kt = 0, slot = 0;
        const std::true_type yes{};
        const std::false_type no{};
        for (; kt + 2 < KT; ++kt) {
            slab(kt, slot, yes, yes);
            slot = slot == 2 ? 0 : slot + 1;
        }
        if (kt + 1 < KT) {
            slab(kt++, slot, yes, no);
            slot = slot == 2 ? 0 : slot + 1;
        }
        slab(kt, slot, no, no);
        // the last matrix instructions retire before anything else reads the accumulators
        asm volatile("s_nop 15\n\ts_nop 15");
    }
};

// A block's place among the units of an item that is cut along K (slices == 1: the whole item).
struct SplitUnit {
    int slices, slice;
    int stride;      // units between consecutive slices of one item
    float* partial;  // slice 0 of this item
    int* counter;    // this item's ticket
};

// Block tile of BM activation rows x BN weight rows over 64-wide K slabs, WAVES_M x WAVES_N waves, on the
// loop above.  One output tile: rows [row0, row0+rows) of expert e times kNCols output columns from n0.
//
// LDS rows are 128 bytes (64 bf16).  They are filled by direct global->LDS loads: one wave-wide load writes
// 1 KB of consecutive LDS (64 lanes x 16 bytes = 8 rows), and each lane chooses WHICH 16-byte piece of its
// row it fetches, so that piece kc of row r lands at position kc ^ ((r >> 1) & 7): with the 64 LDS banks of
// this chip, the 16 lanes that a 16-byte read serves per cycle then fall into 16 different bank groups, for
// the fill as well as for the operand reads.  Lane l reads row (l & 15), piece (l >> 4) of a k-step and ends
// with output columns 4*(l >> 4) .. +3 of activation row (l & 15) of each 16 x 16 sub-tile.
//
// SWIGLU: weight rows [0,BN/2) of the tile come from W_gate, [BN/2,BN) from W_up, for the same BN/2 hidden
// columns; a wave holds matching gate and up columns and applies silu(g)*u itself.
//
// Two shapes are used: 256 x 256 with 2 x 2 waves (128 x 128 per wave) for full-height row tiles, and
// 64 x 256 with 1 x 4 waves (64 x 64 per wave) for the short remainders, where the work is weight streaming.
template <int BM, int BN, int WAVES_M, int WAVES_N, bool SWIGLU>
struct TileConfig16 {
    static constexpr int kBM = BM, kBN = BN;
    static constexpr int kNCols = SWIGLU ? BN / 2 : BN;
    static constexpr int kThreads = 64 * WAVES_M * WAVES_N;
    static constexpr int kLdsBytes = 2 * BM * 128 + 3 * BN * 128;

    static __device__ __forceinline__ void run(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
                                               const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
                                               const int32_t* __restrict__ gather, int e, int row0, int rows, int n0,
                                               int K, int Nout, uint8_t* smem, const SplitUnit& split) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 16, TN = WTN / 16;
    constexpr int A_GROUPS = BM / 8, GROUPS = (BM + BN) / 8;  // eight 128-byte rows per wave-wide load
    constexpr int LOADS = GROUPS / NW, A_LOADS = A_GROUPS / NW, B_LOADS = LOADS - A_LOADS;
    constexpr int B1_FROM = SWIGLU ? A_LOADS + B_LOADS / 2 : LOADS;
    static_assert(GROUPS % NW == 0 && A_GROUPS % NW == 0 && (!SWIGLU || B_LOADS % 2 == 0),
                  "a wave-wide load must not straddle two tensors");
    static_assert(WTM % 32 == 0 && WTN % 16 == 0 && (!SWIGLU || TN % 2 == 0), "wave tile");
    static_assert(B_LOADS < 64, "vmcnt range");

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WAVES_N, wn = wv % WAVES_N;

    // ---- sources of this lane's pieces ----
    // Each descriptor opens the block's own window of a tensor (its activation rows, its weight rows), so
    // 32-bit byte offsets suffice whatever the tensor size; with a gather list the window is the whole
    // unpermuted input, whose size the host checks.
    constexpr int kRsrcFlags = 0x00020000;  // raw buffer of 32-bit words, no swizzle (gfx9 descriptor word 3)
    using FillsT = Fills<LOADS, A_LOADS, B1_FROM>;
    FillsT fills;
    fills.a = __builtin_amdgcn_make_buffer_rsrc((void*)(gather ? A : A + (size_t)row0 * K), 0, -1, kRsrcFlags);
    fills.b0 = __builtin_amdgcn_make_buffer_rsrc((void*)(B0 + ((size_t)e * Nout + n0) * K), 0, -1, kRsrcFlags);
    fills.b1 = SWIGLU ? __builtin_amdgcn_make_buffer_rsrc((void*)(B1 + ((size_t)e * Nout + n0) * K), 0, -1, kRsrcFlags)
                      : fills.b0;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int g = wv + NW * i;          // row group: activation rows first, then weight rows
        const int r = g * 8 + lane / 8;
        const int kc = (lane % 8) ^ ((r >> 1) & 7);
        if (i < A_LOADS) {
            const int rr = r < rows ? r : rows - 1;  // rows past the expert's end repeat its last row
            const uint32_t arow = gather ? (uint32_t)gather[row0 + rr] : (uint32_t)rr;
            fills.voff[i] = (arow * (uint32_t)K + kc * 8) * 2u;
        } else {
            int rb = r - BM;
            if (SWIGLU && rb >= BN / 2) rb -= BN / 2;  // the up-projection rows of the same hidden columns
            fills.voff[i] = ((uint32_t)rb * (uint32_t)K + kc * 8) * 2u;
        }
    }

    // ---- this lane's operand pieces: row (lane & 15) of a sub-tile, piece (lane >> 4) of a k-step ----
    // every sub-tile starts at a multiple of 16 rows, so the piece swizzle (row >> 1) & 7 depends on the
    // lane only and the sub-tiles differ by constant offsets
    const int lr = lane & 15, lk = lane >> 4;
    const int piece0 = (lk ^ ((lr >> 1) & 7)) << 4;
    const int a_lane = (wm * WTM + lr) * 128 + piece0;
    const int b_lane = ((SWIGLU ? wn * (WTN / 2) : wn * WTN) + lr) * 128 + piece0;

    f32x4 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

    // 16-row sub-tiles of this wave that hold rows of the expert, in pairs (wave-uniform); the main loop
    // is specialised on it so that the common full tile carries no conditionals
    int live = (rows - wm * WTM + 31) / 32 * 2;
    live = __builtin_amdgcn_readfirstlane(live < 0 ? 0 : (live > TM ? TM : live));

    using Loop = PipelinedLoop16<BM, BN, NW, TM, TN, WTN, SWIGLU, LOADS, FillsT>;
    static_assert(Loop::LDS_BYTES == kLdsBytes, "LDS size");
    // this block's share of the K slabs: all of them, or slice `split.slice` of `split.slices`
    const int slabs_all = K / 64;
    const int k_first = split.slices > 1 ? (int)((long long)split.slice * slabs_all / split.slices) : 0;
    const int k_end = split.slices > 1 ? (int)((long long)(split.slice + 1) * slabs_all / split.slices) : slabs_all;
    Loop loop{smem, fills, a_lane, b_lane, k_end - k_first, __builtin_amdgcn_readfirstlane(wv), k_first};
    if (live == TM) {
        switch (loop.wv & 3) {
            case 0: loop.template run<TM, 0>(acc); break;
            case 1: loop.template run<TM, 1>(acc); break;
            case 2: loop.template run<TM, 2>(acc); break;
            default: loop.template run<TM, 3>(acc); break;
        }
    } else if (TM > 6 && live == 6)
        loop.template run<(TM > 6 ? 6 : TM)>(acc);
    else if (TM > 4 && live == 4)
        loop.template run<(TM > 4 ? 4 : TM)>(acc);
    else if (TM > 2 && live == 2)
        loop.template run<(TM > 2 ? 2 : TM)>(acc);
    else
        loop.template run<0>(acc);

    // ---- an item cut along K: partial tiles through the workspace, the last unit to finish adds them ----
    // The units of an item may run on different XCDs, whose L2 caches do not see each other's lines.  A fence
    // that writes back and invalidates a whole L2 per unit costs more than the cut saves, so the partial tiles
    // are stored and loaded with device-scope cache policy instead (written through to memory, read around
    // caches that may be stale), each store is acknowledged before the ticket is taken, and the ticket is a
    // device-scope atomic.
    if (split.slices > 1) {
        // a unit's partial tile is stored in register order (fragment, lane): whole 1 KB lines per wave store
        constexpr int FRAGS = TN * TM;
        constexpr int kDeviceScope = 16;  // cache policy bit sc1 of the buffer instructions
        const size_t unit_floats = (size_t)BM * BN;
        typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
        const uint32_t at = (uint32_t)((wv * FRAGS * 64 + lane) * 16);  // + fragment * 1024 bytes
        {
            const __amdgpu_buffer_rsrc_t mine = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(split.partial + (size_t)(split.slice * split.stride) * unit_floats), 0, -1, kRsrcFlags);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    const f32x4 v = acc[i][j];
                    __builtin_amdgcn_raw_buffer_store_b128(*(const u32x4*)&v, mine, at + (i * TM + j) * 1024, 0, kDeviceScope);
                }
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));  // every store of this lane has been acknowledged
        __syncthreads();
        int* ticket = (int*)smem;  // the operand slots are free: the loop's last barrier follows its last read
        if (tid == 0) *ticket = __hip_atomic_fetch_add(split.counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int order = *ticket;
        __syncthreads();
        if (order != split.slices - 1) return;  // another unit of this item finishes later and does the sum
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
        for (int sl = 0; sl < split.slices; ++sl) {  // slice order, whichever unit does it: the same sum every run
            const __amdgpu_buffer_rsrc_t theirs = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(split.partial + (size_t)(sl * split.stride) * unit_floats), 0, -1, kRsrcFlags);
            // up to 32 loads in flight at a time: a load that goes around the caches takes microseconds
            constexpr int BATCH = FRAGS < 32 ? FRAGS : 32;
            static_assert(FRAGS % BATCH == 0, "fragment batches");
#pragma unroll
            for (int g = 0; g < FRAGS; g += BATCH) {
                u32x4 q[BATCH];
#pragma unroll
                for (int t = 0; t < BATCH; ++t)
                    q[t] = __builtin_amdgcn_raw_buffer_load_b128(theirs, at + (g + t) * 1024, 0, kDeviceScope);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < BATCH; ++t) {
                    const f32x4 p = *(const f32x4*)&q[t];
                    const int i = (g + t) / TM, j = (g + t) % TM;
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[i][j][v] += p[v];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- epilogue ----
    // The tile is transposed through LDS (free after the K loop: its last barrier follows the last operand
    // read), because a lane holds 8-byte runs scattered over 16 rows and a wave store of those touches 64
    // cache lines: bf16 rows of OUT_COLS columns, 16-byte piece p of row r at position
    // p ^ (r mod PIECES), then every row leaves as consecutive 16-byte pieces of consecutive lanes.
    constexpr int TNO = SWIGLU ? TN / 2 : TN;
    constexpr int OUT_COLS = kNCols, ROWB = OUT_COLS * 2, PIECES = ROWB / 16;
    static_assert(BM * ROWB <= kLdsBytes, "the output tile must fit in the operand slots");
    static_assert((PIECES & (PIECES - 1)) == 0, "piece swizzle");
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int r = wm * WTM + j * 16 + lr;
        uint8_t* lrow = smem + r * ROWB + (lk & 1) * 8;
        const int sw = r & (PIECES - 1);
#pragma unroll
        for (int i = 0; i < TNO; ++i) {
            const int piece = ((SWIGLU ? wn * (WTN / 2) : wn * WTN) + i * 16) / 8 + (lk >> 1);
            float o[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float g = acc[i][j][v];
                if (SWIGLU) {
                    const float u = acc[i + TN / 2][j][v];
                    o[v] = g * u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.4426950408889634f));
                } else {
                    o[v] = g;
                }
            }
            uint2 pk;
            pk.x = pack_bf16x2(o[0], o[1]);
            pk.y = pack_bf16x2(o[2], o[3]);
            *(uint2*)(lrow + ((piece ^ sw) << 4)) = pk;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < BM * PIECES; idx += kThreads) {
        const int r = idx / PIECES, pc = idx % PIECES;
        if (r < rows) {
            const uint4 v = *(const uint4*)(smem + r * ROWB + ((pc ^ (r & (PIECES - 1))) << 4));
            *(uint4*)(C + (size_t)(row0 + r) * Nout + n0 + pc * 8) = v;
        }
    }
}
};

// Decode a block's position in a list of `total` = tiles x column blocks work items, ordered
// [column group][row tile][column in group].
__device__ inline void decode_item(int logical, int nt, int col_group, int& tile, int& nb) {
    const int per_group = nt * col_group;
    const int cg = logical / per_group, rem = logical - cg * per_group;
    tile = rem / col_group;
    nb = cg * col_group + (rem - tile * col_group);
}

// One launch serves both kinds of tile.  Every XCD (block id mod 8) gets a contiguous eighth of the work, and
// blocks that run together on an XCD share row and weight tiles in its L2.
//
// split_hdr[4] set (see the tile schedule: a long launch that is never cut along K): the blocks walk the list
// that holds both kinds expert by expert, so the short tiles of an expert run next to its big tiles and their
// weight streaming overlaps matrix work.
//
// Otherwise the two lists one after the other: the XCD's eighth of the big items, then its eighth of the short
// ones (longest first).  The last split_hdr[0] big items of an XCD's share run as split_hdr[1] units each; the
// units follow the XCD's whole items in launch order, slice by slice, so that the units that run together read
// the same K range of the tiles they share.
template <class Big, class Small, bool SWIGLU>
__global__ __launch_bounds__(Big::kThreads) void ffn_gemm_bf16_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1,
    uint16_t* __restrict__ C, const int32_t* __restrict__ gather, const TileListArgs L, int K, int Nout,
    int col_group_big, int col_group_small, const int32_t* __restrict__ split_hdr, float* split_partial,
    int32_t* split_counter) {
    static_assert(Big::kThreads == Small::kThreads, "one block size");
    static_assert(Big::kNCols == Small::kNCols, "one column-block width: the joint list is decoded with it");
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int32_t* __restrict__ b_expert = L.b_expert;
    const int32_t* __restrict__ b_row0 = L.b_row0;
    const int32_t* __restrict__ b_rows = L.b_rows;
    const int32_t* __restrict__ s_expert = L.s_expert;
    const int32_t* __restrict__ s_row0 = L.s_row0;
    const int32_t* __restrict__ s_rows = L.s_rows;
    const int cut = split_hdr ? split_hdr[0] : 0, slices = split_hdr ? split_hdr[1] : 1;
    const int cut_s = split_hdr ? split_hdr[2] : 0, slices_s = split_hdr ? split_hdr[3] : 1;
    const int xcd = blockIdx.x & 7;
    int slot = blockIdx.x >> 3;
    int tile, nb;
    const SplitUnit one{1, 0, 0, nullptr, nullptr};
    if (split_hdr && split_hdr[4]) {
        const int nt = *L.u_count;
        const int total = nt * (Nout / Big::kNCols);
        // The last split_hdr[5] items of the order are not dealt out in eighths: whichever XCD has a compute
        // unit free takes the next one (a counter), so that an XCD that runs a few per cent slower than the others
        // (they differ) does not end the launch alone.  Every XCD brings blocks for a quarter of that pool, twice
        // its even share; the ones that find the pool empty leave.
        const int pool = split_hdr[5], fixed = total - pool, chunk = (fixed + 7) >> 3;
        int logical = xcd * chunk + slot;
        if (slot >= chunk) {
            if (slot - chunk >= (pool + 3) >> 2) return;
            int* next = (int*)smem;
            if (threadIdx.x == 0)
                *next = __hip_atomic_fetch_add(split_counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            const int taken = *next;
            __syncthreads();
            if (taken >= pool) return;
            logical = fixed + taken;
        } else if (logical >= fixed) {
            return;
        }
        decode_item(logical, nt, col_group_big, tile, nb);
        const int rows = L.u_rows[tile];
        if (rows >= kShortTileFlag)
            Small::run(A, B0, B1, C, gather, L.u_expert[tile], L.u_row0[tile], rows - kShortTileFlag, nb * Small::kNCols,
                       K, Nout, smem, one);
        else
            Big::run(A, B0, B1, C, gather, L.u_expert[tile], L.u_row0[tile], rows, nb * Big::kNCols, K, Nout, smem, one);
        return;
    }
    const int nt_b = *L.b_count, nt_s = *L.s_count;
    const int total_b = nt_b * (Nout / Big::kNCols), total_s = nt_s * (Nout / Small::kNCols);
    const int chunk_b = (total_b + 7) >> 3, chunk_s = (total_s + 7) >> 3;
    // per XCD: whole big items, the row pieces of big items (see below), whole short items, then the units of the cut
    // big items and of the cut short ones (longest work first, the shortest pieces fill the end)
    const int in_rows = split_hdr ? split_hdr[6] : 0;
    const int whole = chunk_b - cut - in_rows, units = cut * slices, whole_s = chunk_s - cut_s, units_s = cut_s * slices_s;
    constexpr int per_xcd = kFfnSplitUnits / 8;
    if (slot < whole) {
        const int logical = xcd * chunk_b + slot;
        if (logical >= total_b) return;
        decode_item(logical, nt_b, col_group_big, tile, nb);
        Big::run(A, B0, B1, C, gather, b_expert[tile], b_row0[tile], b_rows[tile], nb * Big::kNCols, K, Nout, smem, one);
        return;
    }
    slot -= whole;
    // A GEMM too short in K to be cut there runs the few big items left over after the XCD's last full round as
    // kRowPieces short-tile blocks each (rows 0-63, 64-127, ... of the item): twice the compute-unit time, on
    // compute units that would have idled, in half the item's time.
    constexpr int kRowPieces = Big::kBM / Small::kBM;
    static_assert(Big::kBM % Small::kBM == 0, "a big tile is a whole number of short tiles");
    if (slot < in_rows * kRowPieces) {
        const int idx = slot / kRowPieces, piece = slot - idx * kRowPieces;
        const int logical = xcd * chunk_b + whole + idx;
        if (logical >= total_b) return;
        decode_item(logical, nt_b, col_group_big, tile, nb);
        const int first = piece * Small::kBM, left = b_rows[tile] - first;
        if (left <= 0) return;
        Small::run(A, B0, B1, C, gather, b_expert[tile], b_row0[tile] + first, left < Small::kBM ? left : Small::kBM,
                   nb * Small::kNCols, K, Nout, smem, one);
        return;
    }
    slot -= in_rows * kRowPieces;
    if (slot < whole_s) {
        const int logical = xcd * chunk_s + slot;
        if (logical >= total_s) return;
        decode_item(logical, nt_s, col_group_small, tile, nb);
        Small::run(A, B0, B1, C, gather, s_expert[tile], s_row0[tile], s_rows[tile], nb * Small::kNCols, K, Nout, smem,
                   one);
        return;
    }
    slot -= whole_s;
    if (slot < units) {
        // unit (xcd, slice, idx) keeps its partial tile at unit index xcd * units-per-XCD + slice * cut + idx
        const int slice = slot / cut, idx = slot - slice * cut;
        const int logical = xcd * chunk_b + whole + idx;
        if (logical >= total_b) return;
        decode_item(logical, nt_b, col_group_big, tile, nb);
        const SplitUnit su{slices, slice, cut,
                           split_partial + (size_t)(xcd * per_xcd + idx) * ((size_t)Big::kBM * Big::kBN),
                           split_counter + xcd * per_xcd + idx};
        Big::run(A, B0, B1, C, gather, b_expert[tile], b_row0[tile], b_rows[tile], nb * Big::kNCols, K, Nout, smem, su);
        return;
    }
    slot -= units;
    if (slot < units_s) {
        const int slice = slot / cut_s, idx = slot - slice * cut_s;
        const int logical = xcd * chunk_s + whole_s + idx;
        if (logical >= total_s) return;
        decode_item(logical, nt_s, col_group_small, tile, nb);
        // the short items' partial tiles follow those of the big items
        float* region = split_partial + (size_t)kFfnSplitUnits * kFfnTileM * 256;
        const SplitUnit su{slices_s, slice, cut_s,
                           region + (size_t)(xcd * per_xcd + idx) * ((size_t)Small::kBM * Small::kBN),
                           split_counter + kFfnSplitUnits + xcd * per_xcd + idx};
        Small::run(A, B0, B1, C, gather, s_expert[tile], s_row0[tile], s_rows[tile], nb * Small::kNCols, K, Nout, smem,
                   su);
    }
}

// The three tile lists of a workspace as the kernels take them; joint == false leaves the joint list unwritten
// (the fp32 kernels walk the list of big tiles only).
static TileListArgs tile_list_args(const FfnWorkspace& ws, bool joint) {
    return TileListArgs{ws.big.expert, ws.big.row0,  ws.big.rows,      ws.big.count,       ws.small.expert,
                        ws.small.row0, ws.small.rows, ws.small.count,   ws.big.max_tiles,   ws.small.max_tiles,
                        ws.all.expert, ws.all.row0,  ws.all.rows,      ws.all.count,       joint ? ws.all.max_tiles : 0};
}

static int column_group(int nb_total) {
    for (int g = 4; g > 1; --g)
        if (nb_total % g == 0) return g;
    return 1;
}

template <class Big, class Small, bool SWIGLU>
static void launch_bf16(const void* A, const void* B0, const void* B1, void* C, const int32_t* gather,
                        const FfnWorkspace& ws, int K, int Nout, const int32_t* split_hdr, int32_t* split_counter,
                        hipStream_t st) {
    constexpr int lds = Big::kLdsBytes > Small::kLdsBytes ? Big::kLdsBytes : Small::kLdsBytes;
    auto kern = ffn_gemm_bf16_kernel<Big, Small, SWIGLU>;
    static std::atomic<uint64_t> configured{0};
    once_per_device(configured, [&] {
        (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    const int nb_b = Nout / Big::kNCols, nb_s = Nout / Small::kNCols;
    // items cut along K (or into row pieces) add at most kFfnSplitUnits blocks per list, the pool at the end of the
    // joint order as many blocks as it has items; + 16: both lists are cut into eight whole chunks
    const long long grid =
        (long long)nb_b * ws.big.max_launch + (long long)nb_s * ws.small.max_launch +
        std::max(2 * kFfnSplitUnits, kFfnJointPoolRounds * compute_units()) + 16;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(Big::kThreads), lds, st, (const uint16_t*)A,
                       (const uint16_t*)B0, (const uint16_t*)B1, (uint16_t*)C, gather, tile_list_args(ws, true), K, Nout,
                       column_group(nb_b), column_group(nb_s), split_hdr, ws.split_partial, split_counter);
}

// The arguments of the tile schedule for a descriptor and its workspace layout (host side).
FfnScheduleArgs ffn_schedule_args(const moe_desc_t& d, const FfnWorkspace& ws, int cus) {
    const bool bf16 = d.dtype == MOE_DTYPE_BF16;
    const int K1 = d.d_model, N1 = d.d_hidden, K2 = d.d_hidden, N2 = d.d_model;
    const int bn_down = N2 % 256 == 0 ? 256 : 128;
    auto log2i = [](int v) {
        int sh = 0;
        while ((1 << sh) < v) ++sh;
        return sh;
    };
    FfnScheduleArgs a;
    a.enabled = 1;
    a.E = d.n_experts;
    a.big_sh = log2i(ws.big.tile_m);
    a.small_sh = log2i(ws.small.tile_m);
    a.small_max = ws.small_max;
    a.cus = cus;
    a.L = tile_list_args(ws, bf16);
    // gate/up: a big item covers 128 hidden columns (gate and up rows of them)
    const bool split = bf16;
    a.first = SplitArgs{split ? ws.split_hdr : nullptr, split ? ws.split_counter : nullptr, N1 / 128, N1 / 128, K1 / 64};
    a.second = SplitArgs{split ? ws.split_hdr + kFfnSplitHdr : nullptr, split ? ws.split_counter + 2 * kFfnSplitUnits : nullptr,
                         N2 / bn_down, N2 / bn_down, K2 / 64};
    return a;
}

// What the schedule decides for given per-expert row counts, on the host (moe_ffn_schedule_query).
void ffn_schedule_on_host(const moe_desc_t& d, const FfnWorkspace& ws, const int32_t* expert_count, int cus,
                          int32_t* tiles, int32_t* header) {
    FfnWorkspace layout = ws;
    int32_t hdr_gate_up[kFfnSplitHdr] = {}, hdr_down[kFfnSplitHdr] = {};
    layout.split_hdr = nullptr;  // the headers are written below, not through the workspace
    const FfnScheduleArgs a = ffn_schedule_args(d, layout, cus);
    int nb = 0, ns = 0;
    for (int e = 0; e < d.n_experts; ++e) {
        const ExpertTiles t = expert_tiles(0, expert_count[e], a.big_sh, a.small_sh, a.small_max);
        nb += t.nb;
        ns += t.ns;
    }
    if (d.dtype == MOE_DTYPE_BF16) {
        ffn_schedule_header(nb, ns, a.first.ncol_big, a.first.ncol_small, a.first.slabs, cus, true, true, hdr_gate_up);
        ffn_schedule_header(nb, ns, a.second.ncol_big, a.second.ncol_small, a.second.slabs, cus, true, true, hdr_down);
    }
    tiles[0] = nb;
    tiles[1] = ns;
    for (int i = 0; i < kFfnSplitHdr; ++i) {
        header[i] = hdr_gate_up[i];
        header[kFfnSplitHdr + i] = hdr_down[i];
    }
}

// row_token == nullptr: xp holds the permuted rows.  Otherwise xp is the unpermuted x and row r of the
// plan is fetched from x[row_token[r]] (dispatch fused into the first GEMM's operand fetch).
// schedule_ready: the tile schedule is in the workspace already (built by the drop), no schedule kernel is launched.
hipError_t launch_grouped_ffn(const moe_desc_t& d, const Sizes& s, const FfnWorkspace& ws, const void* xp,
                              const int32_t* row_token, const int32_t* expert_offset, const void* w_gate,
                              const void* w_up, const void* w_down, void* yp, bool schedule_ready, hipStream_t st) {
    (void)s;
    const int K1 = d.d_model, N1 = d.d_hidden, K2 = d.d_hidden, N2 = d.d_model;
    const bool bf16 = d.dtype == MOE_DTYPE_BF16;
    const int bn_down = N2 % 256 == 0 ? 256 : 128;  // d is a multiple of 128 at least: output columns per block
    if (!schedule_ready) {
        ProfileScope prof(MOE_KERNEL_FFN_SCHEDULE, st);
        hipLaunchKernelGGL(ffn_schedule_kernel, dim3(1), dim3(64), 0, st, expert_offset, ffn_schedule_args(d, ws, compute_units()));
    }
    if (bf16) {
        const int32_t* split_gu = ws.split_hdr;
        const int32_t* split_dn = ws.split_hdr + kFfnSplitHdr;
        // full-height row tiles: 256 x 256 blocks; short remainders: 64 x 256 blocks; four waves each
        {
            ProfileScope prof(MOE_KERNEL_FFN_GATE_UP, st);
            launch_bf16<TileConfig16<kFfnTileM, 256, 2, 2, true>, TileConfig16<kFfnTileSmall, 256, 1, 4, true>,
                        true>(xp, w_gate, w_up, ws.hidden, row_token, ws, K1, N1, split_gu, ws.split_counter, st);
        }
        ProfileScope prof(MOE_KERNEL_FFN_DOWN, st);
        if (bn_down == 256)
            launch_bf16<TileConfig16<kFfnTileM, 256, 2, 2, false>,
                        TileConfig16<kFfnTileSmall, 256, 1, 4, false>, false>(ws.hidden, w_down, nullptr, yp, nullptr,
                                                                                    ws, K2, N2, split_dn,
                                                                                    ws.split_counter + 2 * kFfnSplitUnits, st);
        else
            launch_bf16<TileConfig16<kFfnTileM, 128, 2, 2, false>,
                        TileConfig16<kFfnTileSmall, 128, 1, 4, false>, false>(ws.hidden, w_down, nullptr, yp, nullptr,
                                                                                    ws, K2, N2, split_dn,
                                                                                    ws.split_counter + 2 * kFfnSplitUnits, st);
    } else {
        const dim3 g1(((N1 + 15) / 16) * ws.big.max_tiles), g2(((N2 + 15) / 16) * ws.big.max_tiles);
        {
            ProfileScope prof(MOE_KERNEL_FFN_GATE_UP, st);
            hipLaunchKernelGGL((grouped_gemm_f32_kernel<true>), g1, dim3(256), 0, st, (const float*)xp,
                               (const float*)w_gate, (const float*)w_up, (float*)ws.hidden, ws.big.expert, ws.big.row0,
                               ws.big.rows, ws.big.count, row_token, K1, N1);
        }
        ProfileScope prof(MOE_KERNEL_FFN_DOWN, st);
        hipLaunchKernelGGL((grouped_gemm_f32_kernel<false>), g2, dim3(256), 0, st, (const float*)ws.hidden,
                           (const float*)w_down, (const float*)nullptr, (float*)yp, ws.big.expert, ws.big.row0,
                           ws.big.rows, ws.big.count, (const int32_t*)nullptr, K2, N2);
    }
    return hipGetLastError();
}

}  // namespace capmoe
