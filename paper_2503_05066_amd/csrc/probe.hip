// Measured ceiling of the matrix cores, for the benchmark's "fraction of what the chip sustains"
// figure next to the fraction of the published peak (instrumentation, not part of the method).
//
// Every wave issues `iterations` rounds of 8 independent v_mfma_f32_32x32x16_bf16 on register
// operands: no memory traffic, no dependency between consecutive MFMAs, 128 accumulator registers
// as in the layer's GEMM.  The sums are written once at the end so the loop cannot be removed.
#include "common.h"

namespace capmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;

__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iterations) {
    probe_f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    probe_bf16x8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        a[j] = (__bf16)(float)((threadIdx.x + j) & 3);
        b[j] = (__bf16)(float)((threadIdx.x * 3 + j) & 1);
    }
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace capmoe

extern "C" int moe_probe_mfma_bf16(int blocks, int iterations, float* sink, int64_t* flops, void* stream) {
    if (blocks < 1 || blocks > 65536 || iterations < 1 || iterations > (1 << 20) || !sink) return MOE_ERR_INVALID_ARG;
    hipLaunchKernelGGL(capmoe::probe_mfma_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink, iterations);
    if (flops) *flops = (int64_t)blocks * 4 * iterations * 8 * (2ll * 32 * 32 * 16);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}
