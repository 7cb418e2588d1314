// Kernels of the index-driven half of the exchange: every worker's residual taken
// at the leader's index set and summed in a fixed order (arithmetic of the ring
// all-reduce line of Alg. 1), then the sparse SGD update and the clearing of the
// sent residuals (SGD line / Eq. 3, "not Mask" line).
#pragma once

#include "iwp_common.hpp"

namespace iwp {

__global__ __launch_bounds__(BLOCK) void k_gather_sum(ResidualPtrs R, uint32_t W, const uint32_t* __restrict__ idx,
                                                      uint32_t k, float* __restrict__ sum_out) {
    const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
    if (j >= k) return;
    const uint32_t i = idx[j];
    float acc = R.r[0][i];                       // the fold starts from worker 0's value, not from 0
    for (uint32_t p = 1; p < W; ++p) acc = acc + R.r[p][i];
    sum_out[j] = acc;
}

__global__ __launch_bounds__(BLOCK) void k_apply_update(float* __restrict__ w, const uint32_t* __restrict__ idx,
                                                        const float* __restrict__ sum, uint32_t k, float scale,
                                                        ResidualPtrs R, uint32_t W) {
    const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
    if (j >= k) return;
    const uint32_t i = idx[j];
    const float t = scale * sum[j];              // rounded product ...
    w[i] = w[i] + t;                             // ... then rounded sum (contraction is off)
    for (uint32_t p = 0; p < W; ++p) R.r[p][i] = 0.0f;
}

// Whole-step route: the residuals were already gathered into `gathered`
// (row p = worker p's values at the K pairs, leader's row included) and cleared
// while they streamed by, so what is left is the ordered sum over the workers and
// the weight update.
__global__ __launch_bounds__(BLOCK) void k_reduce_update(const float* __restrict__ gathered, uint32_t W, uint64_t K,
                                                         const uint32_t* __restrict__ idx, float* __restrict__ w,
                                                         float scale, float* __restrict__ sum_out) {
    const uint64_t j = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (j >= K) return;
    float acc = gathered[j];
    for (uint32_t p = 1; p < W; ++p) acc = acc + gathered[(size_t)p * K + j];
    sum_out[j] = acc;
    const uint32_t i = idx[j];
    const float t = scale * acc;
    w[i] = w[i] + t;
}

}  // namespace iwp
