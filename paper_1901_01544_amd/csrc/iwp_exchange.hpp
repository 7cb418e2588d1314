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

// Whole-step route: the workers that streamed (and each layer's leader) left their
// values at the K pairs in `gathered` (row p = worker p) and cleared them on the way.
// A worker that does not accumulate (no gradient: bit p of static_mask) streams
// nothing, so unless it leads the pair's layer its value is fetched and cleared
// here, pair by pair.  Then the ordered sum over the workers and the weight update.
__global__ __launch_bounds__(BLOCK) void k_reduce_update(ResidualPtrs R, uint32_t static_mask,
                                                         const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                         const uint32_t* __restrict__ leader,
                                                         const float* __restrict__ gathered, uint32_t W, uint64_t K,
                                                         const uint32_t* __restrict__ idx, float* __restrict__ w,
                                                         float scale, float* __restrict__ sum_out, uint64_t flat_end) {
    const uint64_t j = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (j >= K) return;
    const uint32_t i = idx[j];
    const bool ok = i < flat_end;                // always true for pairs this library wrote
    uint32_t direct = 0;
    if (static_mask) {
        uint32_t lo = 0, hi = n_layers;          // layer of pair j: last row with out_offset <= j
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (layers[mid].out_offset <= j) lo = mid; else hi = mid;
        }
        direct = static_mask & ~(1u << leader_of(leader, lo, W));
    }
    float acc = 0.0f;
    for (uint32_t p = 0; p < W; ++p) {
        float v;
        if ((direct >> p) & 1u) {
            v = ok ? R.r[p][i] : 0.0f;
            if (ok) R.r[p][i] = 0.0f;
        } else {
            v = gathered[(size_t)p * K + j];
        }
        acc = p == 0 ? v : acc + v;
    }
    sum_out[j] = acc;
    if (!ok) return;
    const float t = scale * acc;
    w[i] = w[i] + t;
}

}  // namespace iwp
