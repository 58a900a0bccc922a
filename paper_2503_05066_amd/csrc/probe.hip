// Measured ceiling of the matrix cores, for the benchmark's "fraction of what the chip sustains"
// figure next to the fraction of the published peak (instrumentation, not part of the method).
//
// Every wave repeats the matrix instructions of one k-step of the layer's big GEMM tile on register
// operands: 8 activation x 8 weight fragments, 64 v_mfma_f32_16x16x32_bf16 into 256 accumulator
// registers, no memory traffic, no dependency between consecutive instructions.  The operands are either
// zeros and ones or random bf16 values in (-2, 2): the clock the chip holds under the loop, and with it
// the rate, depends on how many operand bits switch (measured: 2.3 PFLOP/s against 2.06-2.10).  The sums
// are written once at the end so the loop cannot be removed.
#include "common.h"

namespace capmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(4))) float probe_f32x4;

__device__ inline uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// fragment `index` of this lane: random sign, exponent of 0.5 or 1, random mantissa; or 0 / 1
__device__ inline probe_bf16x8 probe_fragment(int index, int random_operands) {
    union {
        probe_bf16x8 v;
        uint16_t u[8];
    } r;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t h = probe_hash((uint32_t)(index * 8 + j) + threadIdx.x * 977u + blockIdx.x * 131071u);
        r.u[j] = random_operands ? (uint16_t)(((h & 1u) << 15) | ((0x7eu + ((h >> 1) & 1u)) << 7) | ((h >> 8) & 0x7fu))
                                 : (uint16_t)((h & 1u) ? 0x3f80u : 0u);
    }
    return r.v;
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iterations, int random_operands) {
    probe_bf16x8 a[8], b[8];
    probe_f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = probe_fragment(i, random_operands);
        b[i] = probe_fragment(100 + i, random_operands);
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    }
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[i], a[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) s += acc[i][j][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace capmoe

extern "C" int moe_probe_mfma_bf16(int blocks, int iterations, int random_operands, float* sink, int64_t* flops,
                                   void* stream) {
    if (blocks < 1 || blocks > 65536 || iterations < 1 || iterations > (1 << 20) || !sink) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(capmoe::probe_mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink, iterations,
                       random_operands != 0);
    if (flops) *flops = (int64_t)blocks * 4 * iterations * 64 * (2ll * 16 * 16 * 32);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}
