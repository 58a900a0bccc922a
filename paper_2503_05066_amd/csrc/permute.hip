// Permutation into expert-major order and the weighted sum of Eq. (2).  Both are pure
// memory movement: every lane moves 16-byte pieces, consecutive lanes touch consecutive
// pieces of a row.
#include "common.h"

namespace capmoe {

// xp[r,:] = x[row_token[r],:] for r < P.  `pieces` = 16-byte pieces per row.
__global__ __launch_bounds__(256) void dispatch_kernel(const uint4* __restrict__ x,
                                                       const int32_t* __restrict__ expert_offset,
                                                       const int32_t* __restrict__ row_token, uint4* __restrict__ xp,
                                                       int E, int pieces, long long max_items) {
    const long long P = expert_offset[E];
    const long long items = P * pieces < max_items ? P * pieces : max_items;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < items; i += (long long)gridDim.x * 256) {
        const long long r = i / pieces;
        const int c = (int)(i - r * pieces);
        xp[i] = x[(long long)row_token[r] * pieces + c];
    }
}

__device__ inline void accumulate_bf16x8(float* acc, const uint4& v, float w) {
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc[2 * i] = fmaf(w, __uint_as_float(u[i] << 16), acc[2 * i]);
        acc[2 * i + 1] = fmaf(w, __uint_as_float(u[i] & 0xffff0000u), acc[2 * i + 1]);
    }
}

__device__ inline uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;  // inputs are finite
}

// y[t,:] = sum over the token's slots (ascending) of row_weight[r] * yp[r,:], fp32 accumulation.
template <bool BF16>
__global__ __launch_bounds__(256) void combine_kernel(const uint4* __restrict__ yp,
                                                      const float* __restrict__ row_weight,
                                                      const int32_t* __restrict__ pair_row, uint4* __restrict__ y,
                                                      long long items, int pieces, int S) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < items; i += (long long)gridDim.x * 256) {
        const long long t = i / pieces;
        const int c = (int)(i - t * pieces);
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        // eight slots at a time: all row indices, then all weights, then all rows are requested before
        // any is used (three dependent memory levels per batch instead of three per slot); the sum
        // still runs in ascending slot order
        for (int s0 = 0; s0 < S; s0 += 8) {
            int r[8];
            float w[8];
            uint4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = s0 + j < S ? pair_row[t * S + s0 + j] : -1;
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = r[j] >= 0 ? row_weight[r[j]] : 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = r[j] >= 0 ? yp[(long long)r[j] * pieces + c] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (r[j] < 0) continue;
                if (BF16) {
                    accumulate_bf16x8(acc, v[j], w[j]);
                } else {
                    acc[0] = fmaf(w[j], __uint_as_float(v[j].x), acc[0]);
                    acc[1] = fmaf(w[j], __uint_as_float(v[j].y), acc[1]);
                    acc[2] = fmaf(w[j], __uint_as_float(v[j].z), acc[2]);
                    acc[3] = fmaf(w[j], __uint_as_float(v[j].w), acc[3]);
                }
            }
        }
        uint4 o;
        if (BF16) {
            o.x = f32_to_bf16_rne(acc[0]) | (f32_to_bf16_rne(acc[1]) << 16);
            o.y = f32_to_bf16_rne(acc[2]) | (f32_to_bf16_rne(acc[3]) << 16);
            o.z = f32_to_bf16_rne(acc[4]) | (f32_to_bf16_rne(acc[5]) << 16);
            o.w = f32_to_bf16_rne(acc[6]) | (f32_to_bf16_rne(acc[7]) << 16);
        } else {
            o.x = __float_as_uint(acc[0]);
            o.y = __float_as_uint(acc[1]);
            o.z = __float_as_uint(acc[2]);
            o.w = __float_as_uint(acc[3]);
        }
        y[i] = o;
    }
}

static int grid_for(long long items) {
    long long g = (items + 255) / 256;
    const long long cap = 256 * 32;  // a few waves per SIMD; the kernels stride over the rest
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

hipError_t launch_dispatch(const moe_desc_t& d, const Sizes& s, const void* x, const int32_t* expert_offset,
                           const int32_t* row_token, void* xp, hipStream_t st) {
    const int pieces = (int)((size_t)d.d_model * s.elem / 16);
    const long long max_items = (long long)s.max_rows * pieces;
    ProfileScope prof(MOE_KERNEL_DISPATCH, st);
    hipLaunchKernelGGL(dispatch_kernel, dim3(grid_for(max_items)), dim3(256), 0, st, (const uint4*)x, expert_offset,
                       row_token, (uint4*)xp, d.n_experts, pieces, max_items);
    return hipGetLastError();
}

hipError_t launch_combine(const moe_desc_t& d, const Sizes& s, const void* yp, const float* row_weight,
                          const int32_t* pair_row, void* y, hipStream_t st) {
    const int pieces = (int)((size_t)d.d_model * s.elem / 16);
    const long long items = (long long)d.n_tokens * pieces;
    ProfileScope prof(MOE_KERNEL_COMBINE, st);
    if (d.dtype == MOE_DTYPE_BF16)
        hipLaunchKernelGGL((combine_kernel<true>), dim3(grid_for(items)), dim3(256), 0, st, (const uint4*)yp, row_weight,
                           pair_row, (uint4*)y, items, pieces, s.slots);
    else
        hipLaunchKernelGGL((combine_kernel<false>), dim3(grid_for(items)), dim3(256), 0, st, (const uint4*)yp,
                           row_weight, pair_row, (uint4*)y, items, pieces, s.slots);
    return hipGetLastError();
}

}  // namespace capmoe
