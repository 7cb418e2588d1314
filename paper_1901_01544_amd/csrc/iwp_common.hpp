// Shared device-side definitions of the gfx950 kernels: tile geometry, the
// importance key, quad (4 consecutive elements per lane) accesses, wavefront and
// workgroup scans, histogram pick and bitmap ranking.  Wavefronts are 64 lanes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/iwp.h"

// No fused multiply-add anywhere: the update is a rounded product followed by a
// rounded sum (Alg. 1 SGD line read as two fp32 operations).
#pragma clang fp contract(off)

namespace iwp {

typedef float v4f __attribute__((ext_vector_type(4)));   // one 128-bit access

// Local accumulation with momentum (Eq. 3): the product is rounded, then the sum
// (contraction is off for the whole library).  m = 1 leaves the product exact, so the
// result is bit for bit the plain r + g.
__device__ __forceinline__ float accum(float r, float g, float m) {
    const float decayed = m * r;
    return decayed + g;
}
__device__ __forceinline__ v4f accum(v4f r, v4f g, float m) {
    const v4f decayed = r * m;
    return decayed + g;
}

constexpr int BLOCK = 256;                         // 4 wavefronts
constexpr int WAVE = 64;
constexpr int VEC = 4;
constexpr uint32_t CHUNK = BLOCK * VEC;            // 1024 elements per workgroup iteration
constexpr uint32_t CHUNKS_PER_TILE = 4;
constexpr uint32_t TILE = CHUNK * CHUNKS_PER_TILE; // 4096 elements: the streaming unit (measured best on MI355X)
constexpr uint32_t GROUP = 8;                      // tiles per super-tile
#ifndef IWP_LGROUP
#define IWP_LGROUP 1                               // build-time tuning knob: -DIWP_LGROUP=1|2|4|8
#endif
constexpr uint32_t LGROUP = IWP_LGROUP;            // tiles that share one LDS histogram in look 1 (divides GROUP).
                                                   // With the first-digit histogram in several copies 1, 2 and 4 measure
                                                   // alike on the model-shaped sets; on a 10^9-element layer 1 streams
                                                   // about 6 % faster than 2
constexpr uint32_t STILE = TILE * GROUP;           // 32768 elements: unit of the leader-side passes
constexpr uint32_t TILE_WORDS = TILE / 32;         // words of a one-bit-per-element tile bitmap

// The 31-bit key (sign bit is always 0) is resolved most-significant digit first:
// 12 bits (exponent + 4 mantissa bits), then 10, then 9.
constexpr int DIGITS = 3;
__host__ __device__ constexpr int digit_shift(int level) { return level == 0 ? 19 : (level == 1 ? 9 : 0); }
__host__ __device__ constexpr int digit_bits(int level) { return level == 0 ? 12 : (level == 1 ? 10 : 9); }
constexpr uint32_t HIST0 = 1u << 12, HIST1 = 1u << 10, HIST2 = 1u << 9;
// A layer's histograms in the workspace: h0_copies copies of the first digit's (look 1 flushes one LDS
// histogram per workgroup with atomics, and atomics on one address serialise at about 20 ns each on this
// chip, so a layer with thousands of workgroups spreads them over several copies), then one of the second
// digit's and one of the third's.
constexpr uint32_t MAX_H0_COPIES = 16;
constexpr uint32_t FLUSHES_PER_COPY = 512;                 // look-1 workgroups that share one copy
__host__ __device__ constexpr uint32_t layer_hist_words(uint32_t copies) { return copies * HIST0 + HIST1 + HIST2; }

constexpr uint32_t RAW_TILE = 0xFFFFFFFFu;        // stage count of a tile whose candidates did not fit its slot
constexpr uint32_t UNIFORM_TILE = 0xFFFFFFFEu;    // stage count of such a tile whose keys are all the same (say, a tile of zero
                                                  // residuals): the key is the slot's only entry, and the later passes handle
                                                  // the tile from its element count instead of reading it again
constexpr uint32_t RESTAGED = 0x40000000u;        // flag on a stage count: look 2 filled this slot again (from b1) after look 1
                                                  // had overflowed it; look 2's reader of look-1 slots skips such tiles
// Entries in a tile's slot for the passes after look 2 (RAW_TILE and UNIFORM_TILE stay what they are).
__device__ __forceinline__ uint32_t staged_entries(uint32_t stage_count) {
    return stage_count >= UNIFORM_TILE ? stage_count : stage_count & ~RESTAGED;
}
constexpr uint32_t NO_STAGE_BIN = 0xFFFFFFFFu;    // LayerState.stage_bin: look 1 stages nothing for this layer
constexpr uint32_t NOT_AN_ELEMENT = 0xFFFFFFFFu;  // key slot of a lane position past the layer's end

struct DevLayer {
    uint64_t offset;       // first element in the flat buffers
    uint64_t slot_begin;   // first entry of the layer's first tile slot in the staging arrays
    uint32_t n;
    uint32_t k;
    uint32_t out_offset;   // first pair in idx_out / val_out
    uint32_t tile_begin;   // first TILE of the layer in the per-worker tile numbering
    uint32_t stile_begin;  // first STILE of the layer
    uint32_t slot_cap;     // staging entries per tile of this layer
    uint32_t mask_begin;   // first 32-bit word of the layer's encoded mask (threshold mode)
    uint32_t hist_begin;   // first word of the layer's histograms
    uint32_t h0_copies;    // copies of the first-digit histogram (a power of two)
    uint32_t pad;
};

// Where digit `level`'s histogram of a layer starts (level 0: the first copy).
__device__ __forceinline__ uint32_t* layer_hist(uint32_t* hist, const DevLayer& L, int level) {
    uint32_t* h = hist + L.hist_begin;
    return level == 0 ? h : (level == 1 ? h + L.h0_copies * HIST0 : h + L.h0_copies * HIST0 + HIST1);
}
__device__ __forceinline__ const uint32_t* layer_hist(const uint32_t* hist, const DevLayer& L, int level) {
    return layer_hist(const_cast<uint32_t*>(hist), L, level);
}

struct LayerState {        // selection state of one layer, lives in the workspace.  Every field has one writer
                           // (one elected workgroup of one kernel) and is read only by later launches.
    uint32_t b1;           // top key digit of the threshold (first pick)
    uint32_t k_rem0;       // rank of the threshold inside that bin (1-based, counted from the largest key)
    uint32_t p22;          // top two digits (second pick)
    uint32_t k_rem1;       // rank inside that 22-bit group
    uint32_t thr;          // the threshold key (third pick, or given by the caller)
    uint32_t n_eq_take;    // ties to keep
    uint32_t stage_bin;    // look 1 copies out every element whose top digit is >= this bin (from a threshold hint)
    uint32_t prestaged;    // set with the first pick: stage_bin <= b1, so look 1's copies are complete
};

struct StageArrays {       // staged candidates, structure of arrays; tile t of a layer owns entries
    uint32_t* key;         // [slot_begin + t * slot_cap, + slot_cap), filled in index order
    uint32_t* idx;         // position inside the layer
    float* val;
};

struct WorkerPtrs {        // passed by value as a kernel argument
    const float* g[IWP_MAX_WORKERS];
    float* r[IWP_MAX_WORKERS];
    float momentum;        // local accumulation is r <- momentum * r + g (Eq. 3); 1 = plain accumulation
};

struct ResidualPtrs {
    float* r[IWP_MAX_WORKERS];
};

struct WorkerList {        // a subset of the workers, by index
    uint32_t n;
    uint8_t id[IWP_MAX_WORKERS];
};

// Importance of one element as an order-preserving integer (Alg. 1 mask line:
// |grad / w|, with eps added to |w| in fp32 before the correctly rounded divide).
__device__ __forceinline__ uint32_t score_key(float r, float w, float eps) {
    float denom = fabsf(w) + eps;
    float s = fabsf(r) / denom;
    return __float_as_uint(s) & 0x7fffffffu;
}

// The worker that leads layer j.  The table lives in device memory, so it cannot
// be checked on the host: an entry that is out of range is read as worker 0, which
// keeps a bad entry from turning into a wild pointer.
__device__ __forceinline__ uint32_t leader_of(const uint32_t* __restrict__ leader, uint32_t j, uint32_t W) {
    const uint32_t l = leader ? leader[j] : 0u;
    return l < W ? l : 0u;
}

// Which layer does tile t (or super-tile t) belong to.  Uniform across the workgroup.
// A table of more than one layer comes from a plan, which stores the answer behind the
// table's sentinel row: one word per tile, then one per super-tile (a binary search over a
// thousand layers is ten dependent loads before a workgroup can issue its first tile load).
template <bool SUPER>
__device__ __forceinline__ uint32_t find_layer(const DevLayer* __restrict__ layers, uint32_t n_layers, uint32_t t) {
    if (n_layers == 1) return 0u;
    const uint32_t* map = reinterpret_cast<const uint32_t*>(layers + n_layers + 1);
    return SUPER ? map[layers[n_layers].tile_begin + t] : map[t];
}

__device__ __forceinline__ bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <bool NT>
__device__ __forceinline__ v4f load_v4(const float* p) {
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return *reinterpret_cast<const v4f*>(p);
}
template <bool NT>
__device__ __forceinline__ void store_v4(float* p, v4f v) {
    if (NT) __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
    else *reinterpret_cast<v4f*>(p) = v;
}

// Four consecutive elements starting at element i of a layer of n elements.
// vec: the layer base is 16-byte aligned, so a whole quad is one 128-bit load.
// Lanes past the end read nothing and get `fill`.  NT: streaming (non-temporal) access for whole quads.
template <bool NT = false>
__device__ __forceinline__ void load_quad(const float* __restrict__ base, uint32_t i, uint32_t n, bool vec,
                                          float (&v)[4], float fill = 0.0f) {
    if (vec && i + 4 <= n) {
        const v4f t = load_v4<NT>(base + i);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = (i + c < n) ? base[i + c] : fill;
    }
}

template <bool NT = false>
__device__ __forceinline__ void store_quad(float* __restrict__ base, uint32_t i, uint32_t n, bool vec, const float (&v)[4]) {
    if (vec && i + 4 <= n) {
        v4f t; t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        store_v4<NT>(base + i, t);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) if (i + c < n) base[i + c] = v[c];
    }
}

// Inclusive scan across the 64 lanes of a wavefront.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int d = 1; d < WAVE; d <<= 1) {
        const uint32_t y = __shfl_up(x, d, WAVE);
        if (lane >= d) x += y;
    }
    return x;
}

// Exclusive scan over the 256 threads of a workgroup; *total receives the sum.
// `slot` (4 words of LDS) must not be reused before the next __syncthreads().
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* slot, uint32_t* total) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    const uint32_t inc = wave_inclusive_scan(x);
    if (lane == WAVE - 1) slot[wave] = inc;
    __syncthreads();
    const uint32_t w0 = slot[0], w1 = slot[1], w2 = slot[2], w3 = slot[3];
    const uint32_t before = (wave > 0 ? w0 : 0) + (wave > 1 ? w1 : 0) + (wave > 2 ? w2 : 0);
    *total = w0 + w1 + w2 + w3;
    return before + inc - x;
}

// Digit pick over a histogram of NB bins (LDS or global): the bin that holds rank
// k_rem counted from the top bin down, and the rank inside that bin.  All 256
// threads call it; the result is broadcast through `sh` (BLOCK + 2 words of LDS).
// Requires sum(hist) >= k_rem >= 1.
template <int NB>
__device__ __forceinline__ void block_pick(const uint32_t* hist, uint32_t k_rem, uint32_t* sh,
                                           uint32_t* bin_out, uint32_t* k_rem_out) {
    constexpr int PER = NB / BLOCK;
    const uint32_t tid = threadIdx.x;
    uint32_t h[PER];
    uint32_t local = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) { h[q] = hist[tid * PER + q]; local += h[q]; }
    __syncthreads();                       // sh may still be in use by a previous call
    sh[tid] = local;
    if (tid == 0) { sh[BLOCK] = 0u; sh[BLOCK + 1] = 1u; }
    __syncthreads();
    for (int d = 1; d < BLOCK; d <<= 1) {  // inclusive suffix sums over the threads
        const uint32_t v = (tid + d < BLOCK) ? sh[tid + d] : 0u;
        __syncthreads();
        sh[tid] += v;
        __syncthreads();
    }
    const uint32_t incl = sh[tid];
    const uint32_t above = incl - local;
    if (above < k_rem && k_rem <= incl) {  // true for exactly one thread
        uint32_t acc = above, bin = tid * PER;
#pragma unroll
        for (int q = PER - 1; q >= 0; --q) {
            if (acc + h[q] >= k_rem) { bin = tid * PER + q; break; }
            acc += h[q];
        }
        sh[BLOCK] = bin;
        sh[BLOCK + 1] = k_rem - acc;
    }
    __syncthreads();
    *bin_out = sh[BLOCK];
    *k_rem_out = sh[BLOCK + 1];
}

// Orders LDS traffic inside one wavefront (the lanes run in lockstep; this makes
// earlier LDS writes and atomics of the wave visible to its later reads).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Wavefront-private version of bitmap_prefix: each lane owns two of the 128 words.
__device__ __forceinline__ void wave_bitmap_prefix(const uint32_t* map, uint32_t* prefix) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint32_t c0 = __popc(map[2 * lane]), c1 = __popc(map[2 * lane + 1]);
    const uint32_t ex = wave_inclusive_scan(c0 + c1) - (c0 + c1);
    prefix[2 * lane] = ex;
    prefix[2 * lane + 1] = ex + c0;
    wave_sync();
}

// One bit per element of a tile.  prefix[w] = number of set bits in words < w.
// Called by all 256 threads after the bitmap is complete (and synchronised).
__device__ __forceinline__ void bitmap_prefix(const uint32_t* map, uint32_t* prefix, uint32_t* slot) {
    const uint32_t tid = threadIdx.x;
    const uint32_t c = tid < TILE_WORDS ? __popc(map[tid]) : 0u;
    uint32_t tot;
    const uint32_t ex = block_exclusive_scan(c, slot, &tot);
    if (tid < TILE_WORDS) prefix[tid] = ex;
    __syncthreads();
}

// Number of set bits strictly below position `local` of the tile.
__device__ __forceinline__ uint32_t bitmap_rank(const uint32_t* map, const uint32_t* prefix, uint32_t local) {
    const uint32_t wd = local >> 5, b = local & 31u;
    return prefix[wd] + __popc(map[wd] & ((1u << b) - 1u));
}

// Copy the elements of one tile whose top key digit is >= bin into the tile's slot,
// in index order.  key[u][q] / val[u][q]: the lane's element q of chunk u (the
// lane's elements are consecutive, chunks follow each other), NOT_AN_ELEMENT past
// the layer's end.  Returns the number of copies, or RAW_TILE if they exceed the
// slot (then nothing is written).  All 256 threads call it; `slot`: 4 words of LDS.
__device__ __forceinline__ uint32_t stage_tile(const uint32_t (&key)[CHUNKS_PER_TILE][4],
                                               const float (&val)[CHUNKS_PER_TILE][4], uint32_t base, uint32_t bin,
                                               uint32_t cap, uint64_t sb, const StageArrays& A, uint32_t* slot) {
    uint32_t c = 0;
#pragma unroll
    for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            c += (key[u][q] != NOT_AN_ELEMENT && (key[u][q] >> digit_shift(0)) >= bin) ? 1u : 0u;
    uint32_t tot;
    uint32_t o = block_exclusive_scan(c, slot, &tot);
    if (tot > cap) return RAW_TILE;
    if (c) {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (key[u][q] != NOT_AN_ELEMENT && (key[u][q] >> digit_shift(0)) >= bin) {
                    A.key[sb + o] = key[u][q];
                    A.idx[sb + o] = base + u * CHUNK + threadIdx.x * VEC + q;
                    A.val[sb + o] = val[u][q];
                    ++o;
                }
    }
    return tot;
}

}  // namespace iwp
