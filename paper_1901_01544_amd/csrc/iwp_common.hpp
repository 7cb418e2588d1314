// Shared device-side definitions of the gfx950 kernels: tile geometry, the
// importance key, quad (4 consecutive elements per lane) loads and the
// wavefront / workgroup scan primitives.  Wavefronts are 64 lanes wide.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/iwp.h"

// No fused multiply-add anywhere: the update is a rounded product followed by a
// rounded sum (Alg. 1 SGD line read as two fp32 operations).
#pragma clang fp contract(off)

namespace iwp {

constexpr int BLOCK = 256;                         // 4 wavefronts
constexpr int WAVE = 64;
constexpr int VEC = 4;                             // one 128-bit access per lane
constexpr uint32_t CHUNK = BLOCK * VEC;            // 1024 elements per workgroup iteration
constexpr uint32_t CHUNKS_PER_TILE = 16;
constexpr uint32_t TILE = CHUNK * CHUNKS_PER_TILE; // 16384 elements: the unit of work and of the ordered scan

// The 31-bit key (sign bit is always 0) is resolved most-significant digit first:
// 11 bits (exponent + 3 mantissa bits), then 10, then 10.
constexpr int DIGITS = 3;
constexpr int HIST_BINS = 2048;                    // bins of the widest digit; per-layer histogram stride
__host__ __device__ constexpr int digit_shift(int level) { return level == 0 ? 20 : (level == 1 ? 10 : 0); }
__host__ __device__ constexpr int digit_bits(int level) { return level == 0 ? 11 : 10; }

struct DevLayer {
    uint64_t offset;      // first element in the flat buffers
    uint32_t n;
    uint32_t k;
    uint32_t out_offset;  // first pair in idx_out / val_out
    uint32_t tile_begin;  // first tile of this layer in the per-worker tile numbering
};

struct LayerState {       // selection state of one layer, lives in the workspace
    uint32_t prefix;      // key bits resolved so far (right-aligned)
    uint32_t k_rem;       // rank still to be found inside the prefix group (1-based)
    uint32_t n_gt;
    uint32_t n_eq_take;
};

struct WorkerPtrs {       // passed by value as a kernel argument
    const float* g[IWP_MAX_WORKERS];
    float* r[IWP_MAX_WORKERS];
};

struct ResidualPtrs {
    float* r[IWP_MAX_WORKERS];
};

// Importance of one element as an order-preserving integer (Alg. 1 mask line:
// |grad / w|, with eps added to |w| in fp32 before the correctly rounded divide).
__device__ __forceinline__ uint32_t score_key(float r, float w, float eps) {
    float denom = fabsf(w) + eps;
    float s = fabsf(r) / denom;
    return __float_as_uint(s) & 0x7fffffffu;
}

// Which layer does tile t (per-worker numbering) belong to: the last row whose
// tile_begin is <= t.  Uniform across the workgroup.
__device__ __forceinline__ uint32_t find_layer(const DevLayer* __restrict__ layers, uint32_t n_layers, uint32_t t) {
    uint32_t lo = 0, hi = n_layers;          // invariant: layers[lo].tile_begin <= t < layers[hi].tile_begin
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (layers[mid].tile_begin <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// Four consecutive elements starting at element i of a layer of n elements.
// vec: the layer base is 16-byte aligned, so a whole quad is one 128-bit load.
// Lanes past the end read nothing and get 0.
__device__ __forceinline__ void load_quad(const float* __restrict__ base, uint32_t i, uint32_t n, bool vec, float (&v)[4]) {
    if (vec && i + 4 <= n) {
        float4 t = *reinterpret_cast<const float4*>(base + i);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = (i + c < n) ? base[i + c] : 0.0f;
    }
}

__device__ __forceinline__ void store_quad(float* __restrict__ base, uint32_t i, uint32_t n, bool vec, const float (&v)[4]) {
    if (vec && i + 4 <= n) {
        *reinterpret_cast<float4*>(base + i) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) if (i + c < n) base[i + c] = v[c];
    }
}

__device__ __forceinline__ bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Inclusive scan across the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        uint32_t y = __shfl_up(x, d, WAVE);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan over the 256 threads of a workgroup; *total receives the sum.
// `slot` (4 words of LDS) must not be reused before the next __syncthreads().
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* slot, uint32_t* total) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    uint32_t inc = wave_inclusive_scan(x);
    if (lane == WAVE - 1) slot[wave] = inc;
    __syncthreads();
    uint32_t w0 = slot[0], w1 = slot[1], w2 = slot[2], w3 = slot[3];
    uint32_t before = (wave > 0 ? w0 : 0) + (wave > 1 ? w1 : 0) + (wave > 2 ? w2 : 0);
    *total = w0 + w1 + w2 + w3;
    return before + inc - x;
}

}  // namespace iwp
