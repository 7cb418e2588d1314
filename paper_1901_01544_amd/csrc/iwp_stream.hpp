// The streaming kernels: Alg. 1's accumulation line (r <- r + g for every worker
// and layer; r <- m * r + g with the momentum of Eq. 3) fused with what can ride along on the same pass over HBM --
//  * on the leader of a layer: the importance of every element and the histogram
//    of its most significant key digit (first look of the selection);
//  * on the other workers, once the leader's index set is known: the gather of
//    the residual at those indices and the clearing of the sent positions
//    (Alg. 1 split lines), so the exchange needs no scattered second pass.
//
// Work unit: one TILE (4096 elements = 4 quads per lane) per workgroup, all loads
// of a tile issued before the first use, non-temporal accesses for data that is
// not read again soon.  This shape measured fastest for a 2-read-1-write stream
// on MI355X (about 6.2 TB/s against 5.3 TB/s for 16K-element tiles and 4.6 TB/s
// for a grid-stride loop).
#pragma once

#include "iwp_common.hpp"

namespace iwp {

// What a leader's workgroup needs besides the data: its LDS histogram, and, when a
// threshold hint makes look 1 copy candidates out, where they go.
struct LeadCtx {
    uint32_t* lh;           // LDS, HIST0 bins
    uint32_t* slot;         // LDS, 2 x 4 words for the scans
    uint32_t stage_bin;     // NO_STAGE_BIN: no staging in look 1
    uint32_t cap;           // slot entries per tile
    uint64_t slot_begin;    // the layer's first slot
    uint32_t* stage_cnt;    // the layer's first tile count
    StageArrays A;
};

// One tile of a plain worker: r <- m * r + g, streaming (non-temporal) accesses.
__device__ __forceinline__ void stream_tile(const float* __restrict__ gl, float* __restrict__ rl, uint32_t n,
                                            uint32_t base, bool vec, float m) {
    const uint32_t tid = threadIdx.x;
    if (vec && base + TILE <= n) {
        v4f rr[CHUNKS_PER_TILE], gg[CHUNKS_PER_TILE];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            rr[u] = load_v4<true>(rl + i);
            gg[u] = load_v4<true>(gl + i);
        }
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            store_v4<true>(rl + i, accum(rr[u], gg[u], m));
        }
    } else {
        // ragged tail of a layer, or a layer whose base is not 16-byte aligned: the same shape, every load of
        // the tile that lies inside the layer issued before the first use
        float rv[CHUNKS_PER_TILE][4], gv[CHUNKS_PER_TILE][4];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (i < n) {
                load_quad<true>(rl, i, n, vec, rv[u]);
                load_quad<true>(gl, i, n, vec, gv[u]);
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (i < n) {
#pragma unroll
                for (int q = 0; q < 4; ++q) rv[u][q] = accum(rv[u][q], gv[u][q], m);
                store_quad<true>(rl, i, n, vec, rv[u]);
            }
        }
    }
}

// One tile of a layer's leader: accumulate (ACC), score every element, histogram
// the top key digit, and with a staging bin copy the candidates into the tile's
// slot.  On large tables everything streams with non-temporal accesses, the leader's
// residual included: the second look comes after the whole first look, far too late for
// any cache (the counters show it fetching every byte from HBM either way), and the
// non-temporal form measured about 10 % faster.  KEEP: on tables small enough for the
// chip's 256 MB memory-side cache the weights (KEEP_W) or the weights and the written
// residual (KEEP_W_AND_R) are accessed with ordinary loads and stores instead, so that
// what touches them again within the step (the ordered write clears the sent positions
// of the residual, the update adds to the weights at them) finds them there: 1-2 % of
// the step on a 25 M-element table, a loss from about 45 M elements on.
constexpr int KEEP_NOTHING = 0, KEEP_W = 1, KEEP_W_AND_R = 2;
template <bool ACC, int KEEP>
__device__ __forceinline__ void lead_tile(const float* __restrict__ gl, float* __restrict__ rl,
                                          const float* __restrict__ wl, uint32_t n, uint32_t lt, bool vec,
                                          float eps, float m, const LeadCtx& C) {
    const uint32_t tid = threadIdx.x;
    const uint32_t base = lt * TILE;
    uint32_t key[CHUNKS_PER_TILE][4];
    float val[CHUNKS_PER_TILE][4];
    if (vec && base + TILE <= n) {
        v4f rr[CHUNKS_PER_TILE], gg[CHUNKS_PER_TILE], ww[CHUNKS_PER_TILE];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            rr[u] = load_v4<true>(rl + i);
            if (ACC) gg[u] = load_v4<true>(gl + i);
            ww[u] = load_v4<(KEEP < KEEP_W)>(wl + i);
        }
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (ACC) {
                rr[u] = accum(rr[u], gg[u], m);
                store_v4<(KEEP < KEEP_W_AND_R)>(rl + i, rr[u]);
            }
            val[u][0] = rr[u].x; val[u][1] = rr[u].y; val[u][2] = rr[u].z; val[u][3] = rr[u].w;
            key[u][0] = score_key(rr[u].x, ww[u].x, eps);
            key[u][1] = score_key(rr[u].y, ww[u].y, eps);
            key[u][2] = score_key(rr[u].z, ww[u].z, eps);
            key[u][3] = score_key(rr[u].w, ww[u].w, eps);
        }
    } else {
        // ragged tail of a layer, or a layer whose base is not 16-byte aligned: the same shape, every load of
        // the tile that lies inside the layer issued before the first use
        float gv[CHUNKS_PER_TILE][4], wv[CHUNKS_PER_TILE][4];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (i < n) {
                load_quad<true>(rl, i, n, vec, val[u]);
                if (ACC) load_quad<true>(gl, i, n, vec, gv[u]);
                load_quad<true>(wl, i, n, vec, wv[u], 1.0f);
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (ACC && i < n) {
#pragma unroll
                for (int q = 0; q < 4; ++q) val[u][q] = accum(val[u][q], gv[u][q], m);
                store_quad<true>(rl, i, n, vec, val[u]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) key[u][q] = (i + q < n) ? score_key(val[u][q], wv[u][q], eps) : NOT_AN_ELEMENT;
        }
    }
    // zero scores (zero residuals: a layer's untouched part) are counted in a register and added once per
    // wavefront: a tile of zeros would otherwise be 4096 atomics on one LDS word
    uint32_t zeros = 0;
#pragma unroll
    for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (key[u][q] == 0u) ++zeros;
            else if (key[u][q] != NOT_AN_ELEMENT) atomicAdd(&C.lh[key[u][q] >> digit_shift(0)], 1u);
        }
    if (__any(zeros != 0)) {
#pragma unroll
        for (int d = WAVE / 2; d > 0; d >>= 1) zeros += __shfl_xor(zeros, d, WAVE);
        if ((tid & (WAVE - 1)) == 0) atomicAdd(&C.lh[0], zeros);
    }
    if (C.stage_bin != NO_STAGE_BIN) {                      // uniform
        const uint32_t cnt = stage_tile(key, val, base, C.stage_bin, C.cap, C.slot_begin + (uint64_t)lt * C.cap, C.A,
                                        C.slot + (lt & 1u) * 4u);
        if (tid == 0) C.stage_cnt[lt] = cnt;
    }
}

// The leader's share of one group (up to LGROUP tiles of the same layer):
// one LDS histogram of the top digit for the whole group, flushed once.
template <int KEEP>
__device__ __forceinline__ void leader_group(const float* gp, float* rp, const float* __restrict__ w, const DevLayer& L,
                                             uint32_t first_tile /*in layer*/, uint32_t group_tiles, float eps, float m,
                                             LeadCtx& C, uint32_t* __restrict__ ghist) {
    for (uint32_t b = threadIdx.x; b < HIST0; b += BLOCK) C.lh[b] = 0u;
    __syncthreads();
    float* rl = rp + L.offset;
    const float* gl = gp ? gp + L.offset : nullptr;
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl) && (!gp || is_aligned16(gl));
    const uint32_t ntiles = (L.n + TILE - 1) / TILE;
    const uint32_t last = min(first_tile + group_tiles, ntiles);
    for (uint32_t t = first_tile; t < last; ++t) {
        if (gp) lead_tile<true, KEEP>(gl, rl, wl, L.n, t, vec, eps, m, C);
        else lead_tile<false, KEEP>(gl, rl, wl, L.n, t, vec, eps, m, C);
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < HIST0; b += BLOCK) {
        const uint32_t v = C.lh[b];
        if (v) atomicAdd(&ghist[b], v);
    }
}

__device__ __forceinline__ LeadCtx lead_ctx(uint32_t* lh, uint32_t* slot, const DevLayer& L, const LayerState* state,
                                            uint32_t j, uint32_t* stage_cnt, const StageArrays& A) {
    LeadCtx C;
    C.lh = lh;
    C.slot = slot;
    C.stage_bin = state[j].stage_bin;
    C.cap = L.slot_cap;
    C.slot_begin = L.slot_begin;
    C.stage_cnt = stage_cnt + L.tile_begin;
    C.A = A;
    return C;
}

// Every worker that is not the leader of the tile's layer (and every worker of a layer
// without selection): plain accumulation, W * tiles workgroups, worker-major.  A worker
// without a gradient pointer is not accumulated.  The leaders go through k_leader_pass.
__global__ __launch_bounds__(BLOCK) void k_accumulate_rest(WorkerPtrs P, const DevLayer* __restrict__ layers,
                                                           uint32_t n_layers, uint32_t tiles,
                                                           const uint32_t* __restrict__ leader, uint32_t W) {
    const uint32_t p = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - p * tiles;
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const float* gp = P.g[p];
    if (!gp || (L.k > 0 && leader_of(leader, j, W) == p)) return;
    float* rl = P.r[p] + L.offset;
    const float* gl = gp + L.offset;
    stream_tile(gl, rl, L.n, (t - L.tile_begin) * TILE, is_aligned16(rl) && is_aligned16(gl), P.momentum);
}

// Leaders only: one workgroup per group of LG tiles of every layer with k > 0.  The grid:
// with LG == 1 one workgroup per tile of the table, otherwise GROUP / LG per super-tile (some of them past the end
// of a short layer).
template <uint32_t LG, int KEEP>
__global__ __launch_bounds__(BLOCK) void k_leader_pass(WorkerPtrs P, const float* __restrict__ w,
                                                       const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                       const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                       uint32_t* __restrict__ hist,
                                                       const LayerState* __restrict__ state,
                                                       uint32_t* __restrict__ stage_cnt, StageArrays A) {
    __shared__ uint32_t lh[HIST0];
    __shared__ uint32_t slot[8];
    uint32_t j, first;
    if (LG == 1) {
        j = find_layer<false>(layers, n_layers, blockIdx.x);
    } else {
        j = find_layer<true>(layers, n_layers, blockIdx.x / (GROUP / LG));
    }
    const DevLayer L = layers[j];
    if (L.k == 0) return;
    if (LG == 1) {
        first = blockIdx.x - L.tile_begin;
    } else {
        constexpr uint32_t SUB = GROUP / LG;                 // workgroups per super-tile
        first = (blockIdx.x / SUB - L.stile_begin) * GROUP + (blockIdx.x % SUB) * LG;
        if (first * TILE >= L.n) return;
    }
    const uint32_t p = leader_of(leader, j, W);
    LeadCtx C = lead_ctx(lh, slot, L, state, j, stage_cnt, A);
    // consecutive workgroups of a layer flush into different copies of its first-digit histogram
    uint32_t* h0 = layer_hist(hist, L, 0) + (size_t)((first / LG) & (L.h0_copies - 1u)) * HIST0;
    leader_group<KEEP>(P.g[p], P.r[p], w, L, first, LG, eps, P.momentum, C, h0);
}

// The other workers, after the leader's pairs are known: accumulate, and where the
// tile holds sent positions, copy the accumulated value into the worker's row of
// the gather matrix and leave +0 behind.  tile_out[t] = position (inside the
// layer's pairs) of the first pair that falls into tile t; the pairs are ascending,
// so a tile's pairs are contiguous.  `acc`: the workers that accumulate (have a
// gradient); the grid is acc.n * tiles.
__global__ __launch_bounds__(BLOCK) void k_follow_gather(WorkerPtrs P, WorkerList acc, const DevLayer* __restrict__ layers,
                                                         uint32_t n_layers, uint32_t tiles,
                                                         const uint32_t* __restrict__ leader, uint32_t W,
                                                         const uint32_t* __restrict__ idx,
                                                         const uint32_t* __restrict__ tile_out,
                                                         float* __restrict__ gathered, uint64_t K) {
    __shared__ uint32_t map[TILE_WORDS], pre[TILE_WORDS], slot[4];
    const uint32_t tid = threadIdx.x;
    const uint32_t a = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - a * tiles;
    const uint32_t p = acc.id[a];
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const bool has_sel = L.k > 0;
    if (has_sel && leader_of(leader, j, W) == p) return;       // done by the leader pass
    const uint32_t lt = t - L.tile_begin;
    const uint32_t base = lt * TILE;
    const float* gp = P.g[p];
    float* rl = P.r[p] + L.offset;
    uint32_t lo = 0, cnt = 0;
    if (has_sel) {
        const uint32_t ntiles = (L.n + TILE - 1) / TILE;
        // positions are clamped to the layer's k pairs: never index outside idx / the gather row
        lo = min(tile_out[t], L.k);
        const uint32_t hi = (lt + 1 < ntiles) ? min(tile_out[t + 1], L.k) : L.k;
        cnt = hi > lo ? min(hi - lo, TILE) : 0u;
    }
    const uint32_t* ix = idx + L.out_offset + lo;
    float* go = gathered + (size_t)p * K + L.out_offset + lo;
    const uint32_t first = (uint32_t)L.offset + base;           // flat position of the tile's first element
    const float* gl = gp + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(gl);
    const bool full = vec && base + TILE <= L.n;
    // the tile's loads go out first; the bitmap of sent positions is built while they are in flight
    float rv[CHUNKS_PER_TILE][4], gv[CHUNKS_PER_TILE][4];      // one set of registers for both forms of the tile
    if (full) {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            const v4f a = load_v4<true>(rl + i);
            const v4f b = load_v4<true>(gl + i);
            rv[u][0] = a.x; rv[u][1] = a.y; rv[u][2] = a.z; rv[u][3] = a.w;
            gv[u][0] = b.x; gv[u][1] = b.y; gv[u][2] = b.z; gv[u][3] = b.w;
        }
    } else {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (i < L.n) {
                load_quad<true>(rl, i, L.n, vec, rv[u]);
                load_quad<true>(gl, i, L.n, vec, gv[u]);
            }
        }
    }
    if (cnt) {                                                   // uniform
        if (tid < TILE_WORDS) map[tid] = 0u;
        __syncthreads();
        for (uint32_t e = tid; e < cnt; e += BLOCK) {
            const uint32_t loc = ix[e] - first;
            if (loc < TILE) atomicOr(&map[loc >> 5], 1u << (loc & 31u));
        }
        __syncthreads();
        bitmap_prefix(map, pre, slot);
    }
    if (full) {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t loc = u * CHUNK + tid * VEC;
#pragma unroll
            for (int q = 0; q < 4; ++q) rv[u][q] = accum(rv[u][q], gv[u][q], P.momentum);
            const uint32_t nib = cnt ? (map[loc >> 5] >> (loc & 31u)) & 0xFu : 0u;
            if (nib) {
                uint32_t rank = bitmap_rank(map, pre, loc);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if ((nib >> q) & 1u) { go[rank++] = rv[u][q]; rv[u][q] = 0.0f; }
            }
            v4f out; out.x = rv[u][0]; out.y = rv[u][1]; out.z = rv[u][2]; out.w = rv[u][3];
            store_v4<true>(rl + base + loc, out);
        }
    } else {
        // ragged tail of a layer, or a layer whose base is not 16-byte aligned (loaded above)
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t loc = u * CHUNK + tid * VEC;
            const uint32_t i = base + loc;
            if (i < L.n) {
                const uint32_t nib = cnt ? (map[loc >> 5] >> (loc & 31u)) & 0xFu : 0u;
                uint32_t rank = nib ? bitmap_rank(map, pre, loc) : 0u;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    rv[u][q] = accum(rv[u][q], gv[u][q], P.momentum);
                    if ((nib >> q) & 1u) { go[rank++] = rv[u][q]; rv[u][q] = 0.0f; }
                }
                store_quad<true>(rl, i, L.n, vec, rv[u]);
            }
        }
    }
}

}  // namespace iwp
