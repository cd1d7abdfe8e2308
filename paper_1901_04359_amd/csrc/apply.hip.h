// The step right after the hot path: the sparse model update of Algorithm 4 line 11,
// W_i = W_{i-1} - eta * G~_i over the k global entries, and the dense gMask that
// Algorithm 3 lines 20-22 return.
#pragma once
#include "common.hip.h"

namespace gtopk {

// weights[c][g_idx[t]] -= lr * g_val[t]: one fp32 multiply, then one fp32 subtract
// (no fused multiply-add: the library is built with -ffp-contract=off).
__global__ __launch_bounds__(kBlock) void k_apply_update(
        float* __restrict__ weights, uint32_t m, int64_t stride, uint32_t k,
        const uint32_t* __restrict__ g_idx, const float* __restrict__ g_val, float lr) {
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = g_idx[t];
    if (i >= m) return;                    // not a valid set: nothing is written outside the row
    float* w = weights + (int64_t)blockIdx.y * stride + i;
    const float p = lr * g_val[t];
    *w = *w - p;
}

// mask[i] = 0 for i in [0, m), 16 bytes per thread where they are aligned and whole
__global__ void k_mask_clear(uint8_t* __restrict__ mask, uint64_t m) {
    const uint64_t step = (uint64_t)gridDim.x * blockDim.x * 16;
    for (uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 16; i < m; i += step) {
        if (i + 16 <= m) {
            *reinterpret_cast<uint4*>(mask + i) = make_uint4(0u, 0u, 0u, 0u);
        } else {
            for (uint64_t j = i; j < m; ++j) mask[j] = 0;
        }
    }
}

__global__ __launch_bounds__(kBlock) void k_mask_set(uint8_t* __restrict__ mask, uint32_t m, uint32_t k,
                                                     const uint32_t* __restrict__ g_idx) {
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t < k && g_idx[t] < m) mask[g_idx[t]] = 1;
}

}  // namespace gtopk
