// Kernels of the per-layer compression: fused residual accumulation + importance
// + first-digit histogram, radix-select refinement, ordered stream compaction.
// All of them are segmented: one launch covers every layer of a layer table.
//
// Tile numbering: a worker's layers are cut into tiles of TILE elements; tile t
// of the per-worker numbering belongs to the layer found by find_layer().  The
// accumulate kernel runs W * tiles workgroups (worker-major), the selection
// kernels run `tiles` workgroups and read the residual of each layer's leader.
#pragma once

#include "iwp_common.hpp"

namespace iwp {

// ---------------------------------------------------------------------------
// Workspace initialisation.  Zeroes the histograms with vector stores (a fill
// kernel rather than a memset node, so the call sequence can be graph-captured)
// and, for the single-layer entry points, writes the one-row layer table.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_init(uint32_t* __restrict__ hist, uint64_t hist_words,
                                                DevLayer* __restrict__ single_table, uint32_t n, uint32_t k) {
    const uint64_t stride = (uint64_t)gridDim.x * BLOCK;
    for (uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x; i < hist_words; i += stride) hist[i] = 0u;
    if (single_table && blockIdx.x == 0 && threadIdx.x == 0) {
        DevLayer row;
        row.offset = 0; row.n = n; row.k = k; row.out_offset = 0; row.tile_begin = 0;
        single_table[0] = row;
        row.n = 0; row.k = 0; row.tile_begin = (n + TILE - 1) / TILE;   // sentinel: total tile count
        single_table[1] = row;
    }
}

// The worker that leads layer j, or W (= nobody) if the table entry is out of
// range: such a layer is accumulated but never scored, so a bad entry cannot turn
// into a wild pointer.
__device__ __forceinline__ uint32_t leader_of(const uint32_t* __restrict__ leader, uint32_t j, uint32_t W) {
    const uint32_t l = leader ? leader[j] : 0u;
    return l < W ? l : W;
}

// LDS histogram -> the layer's global histogram; only non-empty bins are sent.
template <int NB>
__device__ __forceinline__ void flush_hist(const uint32_t* lh, uint32_t* __restrict__ gh) {
    for (int b = threadIdx.x; b < NB; b += BLOCK) {
        uint32_t v = lh[b];
        if (v) atomicAdd(&gh[b], v);
    }
}

// ---------------------------------------------------------------------------
// Look 1.  Alg. 1 accumulation line (r <- r + g, every worker, every layer) fused
// with the mask line's importance on the leader of the layer, whose keys feed the
// histogram of the most significant digit.  Streaming: 8 B read + 4 B written per
// element on a plain worker, + 4 B (w) on the leader.
// ---------------------------------------------------------------------------
template <bool ACC, bool LEAD>
__device__ __forceinline__ void accumulate_tile(const float* __restrict__ gl, float* __restrict__ rl,
                                                const float* __restrict__ wl, uint32_t n, uint32_t base,
                                                float eps, uint32_t* lh) {
    const bool vec = is_aligned16(rl) && (!ACC || is_aligned16(gl)) && (!LEAD || is_aligned16(wl));
    const uint32_t tid = threadIdx.x;
    if (vec && base + TILE <= n) {
        // full tile: 128-bit accesses, loads of four iterations in flight before use
        constexpr int U = 4;
#pragma unroll 1
        for (uint32_t c = 0; c < CHUNKS_PER_TILE; c += U) {
            float4 rr[U], gg[U], ww[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t i = base + (c + u) * CHUNK + tid * VEC;
                rr[u] = *reinterpret_cast<const float4*>(rl + i);
                if (ACC) gg[u] = *reinterpret_cast<const float4*>(gl + i);
                if (LEAD) ww[u] = *reinterpret_cast<const float4*>(wl + i);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t i = base + (c + u) * CHUNK + tid * VEC;
                if (ACC) {
                    rr[u].x = rr[u].x + gg[u].x; rr[u].y = rr[u].y + gg[u].y;
                    rr[u].z = rr[u].z + gg[u].z; rr[u].w = rr[u].w + gg[u].w;
                    *reinterpret_cast<float4*>(rl + i) = rr[u];
                }
                if (LEAD) {
                    atomicAdd(&lh[score_key(rr[u].x, ww[u].x, eps) >> digit_shift(0)], 1u);
                    atomicAdd(&lh[score_key(rr[u].y, ww[u].y, eps) >> digit_shift(0)], 1u);
                    atomicAdd(&lh[score_key(rr[u].z, ww[u].z, eps) >> digit_shift(0)], 1u);
                    atomicAdd(&lh[score_key(rr[u].w, ww[u].w, eps) >> digit_shift(0)], 1u);
                }
            }
        }
    } else {
        // ragged tail of a layer, or a layer whose base is not 16-byte aligned
        for (uint32_t c = 0; c < CHUNKS_PER_TILE; ++c) {
            const uint32_t i = base + c * CHUNK + tid * VEC;
            if (i >= n) break;
            float rv[4], gv[4], wv[4];
            load_quad(rl, i, n, vec, rv);
            if (ACC) {
                load_quad(gl, i, n, vec, gv);
#pragma unroll
                for (int q = 0; q < 4; ++q) rv[q] = rv[q] + gv[q];
                store_quad(rl, i, n, vec, rv);
            }
            if (LEAD) {
                load_quad(wl, i, n, vec, wv);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (i + q < n) atomicAdd(&lh[score_key(rv[q], wv[q], eps) >> digit_shift(0)], 1u);
            }
        }
    }
}

__global__ __launch_bounds__(BLOCK) void k_accumulate_hist(WorkerPtrs P, const float* __restrict__ w,
                                                           const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                           uint32_t tiles, const uint32_t* __restrict__ leader,
                                                           uint32_t W, float eps, uint32_t* __restrict__ hist) {
    __shared__ uint32_t lh[HIST_BINS];
    const uint32_t p = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - p * tiles;
    const uint32_t j = find_layer(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t base = (t - L.tile_begin) * TILE;
    const float* gp = P.g[p];
    float* rp = P.r[p];
    const bool lead = L.k > 0 && leader_of(leader, j, W) == p;
    if (!gp && !lead) return;
    if (lead) {
        for (int b = threadIdx.x; b < HIST_BINS; b += BLOCK) lh[b] = 0u;
        __syncthreads();
    }
    float* rl = rp + L.offset;
    const float* gl = gp ? gp + L.offset : nullptr;
    const float* wl = w + L.offset;
    if (lead) {
        if (gp) accumulate_tile<true, true>(gl, rl, wl, L.n, base, eps, lh);
        else accumulate_tile<false, true>(gl, rl, wl, L.n, base, eps, lh);
        __syncthreads();
        flush_hist<HIST_BINS>(lh, hist + (size_t)j * HIST_BINS);
    } else {
        accumulate_tile<true, false>(gl, rl, wl, L.n, base, eps, lh);
    }
}

// ---------------------------------------------------------------------------
// Digit pick: from the layer's histogram of the current digit, find the bin that
// holds rank k_rem (counting from the top), extend the key prefix by it and
// reduce k_rem to the rank inside that bin.  One workgroup per layer.  The
// histogram is handed back zeroed for the next digit.  After the last digit the
// prefix is the exact k-th largest key and k_rem the tie quota.
// ---------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(BLOCK) void k_pick(const DevLayer* __restrict__ layers, uint32_t* __restrict__ hist,
                                                LayerState* __restrict__ state, iwp_threshold* __restrict__ thr_out) {
    constexpr int NB = 1 << digit_bits(LEVEL);
    constexpr int PER = NB / BLOCK;
    __shared__ uint32_t sums[BLOCK];
    const uint32_t j = blockIdx.x;
    const DevLayer L = layers[j];
    if (L.k == 0) return;
    const uint32_t tid = threadIdx.x;
    const uint32_t k_rem = LEVEL == 0 ? L.k : state[j].k_rem;
    const uint32_t prefix = LEVEL == 0 ? 0u : state[j].prefix;
    uint32_t* gh = hist + (size_t)j * HIST_BINS;
    uint32_t h[PER];
    uint32_t local = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        h[q] = gh[tid * PER + q];
        gh[tid * PER + q] = 0u;
        local += h[q];
    }
    // inclusive suffix sums over the threads (thread t: bins of threads t..255)
    sums[tid] = local;
    __syncthreads();
    for (int d = 1; d < BLOCK; d <<= 1) {
        uint32_t v = (tid + d < BLOCK) ? sums[tid + d] : 0u;
        __syncthreads();
        sums[tid] += v;
        __syncthreads();
    }
    const uint32_t incl = sums[tid];
    const uint32_t above = incl - local;
    if (above < k_rem && k_rem <= incl) {     // true for exactly one thread
        uint32_t acc = above;
        uint32_t bin = tid * PER;
#pragma unroll
        for (int q = PER - 1; q >= 0; --q) {
            if (acc + h[q] >= k_rem) { bin = tid * PER + q; break; }
            acc += h[q];
        }
        LayerState st;
        st.prefix = (prefix << digit_bits(LEVEL)) | bin;
        st.k_rem = k_rem - acc;
        st.n_gt = L.k - st.k_rem;
        st.n_eq_take = st.k_rem;
        state[j] = st;
        if (LEVEL == DIGITS - 1 && thr_out) {
            iwp_threshold th;
            th.key = st.prefix; th.n_gt = st.n_gt; th.n_eq_take = st.n_eq_take;
            thr_out[j] = th;
        }
    }
}

// Threshold records supplied by the caller -> selection state (compact_pairs).
__global__ __launch_bounds__(BLOCK) void k_load_thresholds(const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                           const iwp_threshold* __restrict__ thr,
                                                           LayerState* __restrict__ state) {
    const uint32_t j = blockIdx.x * BLOCK + threadIdx.x;
    if (j >= n_layers || layers[j].k == 0) return;
    LayerState st;
    st.prefix = thr[j].key; st.k_rem = thr[j].n_eq_take; st.n_gt = thr[j].n_gt; st.n_eq_take = thr[j].n_eq_take;
    state[j] = st;
}

// ---------------------------------------------------------------------------
// Refinement look: histogram of digit LEVEL over the elements of the leader's
// residual whose higher digits equal the prefix found so far.
// ---------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(BLOCK) void k_refine_hist(ResidualPtrs R, const float* __restrict__ w,
                                                       const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                       const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                       const LayerState* __restrict__ state,
                                                       uint32_t* __restrict__ hist) {
    constexpr int NB = 1 << digit_bits(LEVEL);
    __shared__ uint32_t lh[NB];
    const uint32_t t = blockIdx.x;
    const uint32_t j = find_layer(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t lead = leader_of(leader, j, W);
    if (L.k == 0 || lead == W) return;
    const uint32_t prefix = state[j].prefix;
    const uint32_t base = (t - L.tile_begin) * TILE;
    const float* rl = R.r[lead] + L.offset;
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl);
    for (int b = threadIdx.x; b < NB; b += BLOCK) lh[b] = 0u;
    __syncthreads();
    for (uint32_t c = 0; c < CHUNKS_PER_TILE; ++c) {
        const uint32_t i = base + c * CHUNK + threadIdx.x * VEC;
        if (i >= L.n) break;
        float rv[4], wv[4];
        load_quad(rl, i, L.n, vec, rv);
        load_quad(wl, i, L.n, vec, wv);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t key = score_key(rv[q], wv[q], eps);
            if (i + q < L.n && (key >> digit_shift(LEVEL - 1)) == prefix)
                atomicAdd(&lh[(key >> digit_shift(LEVEL)) & (NB - 1)], 1u);
        }
    }
    __syncthreads();
    flush_hist<NB>(lh, hist + (size_t)j * HIST_BINS);
}

// ---------------------------------------------------------------------------
// Ordered compaction, part 1: per tile, how many keys lie above the threshold and
// how many equal it.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_tile_count(ResidualPtrs R, const float* __restrict__ w,
                                                      const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                      const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                      const LayerState* __restrict__ state,
                                                      uint2* __restrict__ counts) {
    __shared__ uint32_t cnt[2];
    const uint32_t t = blockIdx.x;
    const uint32_t j = find_layer(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t lead = leader_of(leader, j, W);
    if (L.k == 0 || lead == W) return;
    const uint32_t thr = state[j].prefix;
    const uint32_t base = (t - L.tile_begin) * TILE;
    const float* rl = R.r[lead] + L.offset;
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl);
    if (threadIdx.x < 2) cnt[threadIdx.x] = 0u;
    __syncthreads();
    uint32_t gt = 0, eq = 0;
    for (uint32_t c = 0; c < CHUNKS_PER_TILE; ++c) {
        const uint32_t i = base + c * CHUNK + threadIdx.x * VEC;
        if (i >= L.n) break;
        float rv[4], wv[4];
        load_quad(rl, i, L.n, vec, rv);
        load_quad(wl, i, L.n, vec, wv);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t key = score_key(rv[q], wv[q], eps);
            const bool valid = i + q < L.n;
            gt += (valid && key > thr) ? 1u : 0u;
            eq += (valid && key == thr) ? 1u : 0u;
        }
    }
    if (gt) atomicAdd(&cnt[0], gt);
    if (eq) atomicAdd(&cnt[1], eq);
    __syncthreads();
    if (threadIdx.x == 0) counts[t] = make_uint2(cnt[0], cnt[1]);
}

// Part 2: exclusive prefix of the tile counts inside each layer, in tile order.
__global__ __launch_bounds__(BLOCK) void k_tile_scan(const DevLayer* __restrict__ layers, uint2* __restrict__ counts) {
    __shared__ uint32_t slot_g[4], slot_e[4];
    const uint32_t j = blockIdx.x;
    if (layers[j].k == 0) return;
    const uint32_t tb = layers[j].tile_begin;
    const uint32_t te = tb + (layers[j].n + TILE - 1) / TILE;
    uint32_t G = 0, E = 0;
    for (uint32_t b = tb; b < te; b += BLOCK) {
        const uint32_t t = b + threadIdx.x;
        uint2 v = (t < te) ? counts[t] : make_uint2(0u, 0u);
        uint32_t tot_g, tot_e;
        const uint32_t ex_g = block_exclusive_scan(v.x, slot_g, &tot_g);
        const uint32_t ex_e = block_exclusive_scan(v.y, slot_e, &tot_e);
        if (t < te) counts[t] = make_uint2(G + ex_g, E + ex_e);
        G += tot_g;
        E += tot_e;
        __syncthreads();
    }
}

// Part 3: write the pairs.  An element above the threshold goes to position
// (#above before it) + min(#equal before it, quota); an element equal to the
// threshold is kept iff fewer than `quota` equal elements precede it.  Positions
// are counted in index order, so the output is ascending and ties go to the
// lowest indices (Alg. 1 split: the sent part is the residual itself).
__global__ __launch_bounds__(BLOCK) void k_compact_write(ResidualPtrs R, const float* __restrict__ w,
                                                         const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                         const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                         const LayerState* __restrict__ state,
                                                         const uint2* __restrict__ counts,
                                                         uint32_t* __restrict__ idx_out, float* __restrict__ val_out) {
    __shared__ uint32_t slot[2][4];
    const uint32_t t = blockIdx.x;
    const uint32_t j = find_layer(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t lead = leader_of(leader, j, W);
    if (L.k == 0 || lead == W) return;
    const uint32_t thr = state[j].prefix;
    const uint32_t quota = state[j].n_eq_take;
    const uint32_t base = (t - L.tile_begin) * TILE;
    const float* rl = R.r[lead] + L.offset;
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl);
    uint32_t* io = idx_out + L.out_offset;
    float* vo = val_out + L.out_offset;
    uint32_t G = counts[t].x, E = counts[t].y;
    for (uint32_t c = 0; c < CHUNKS_PER_TILE; ++c) {
        const uint32_t cbase = base + c * CHUNK;
        if (cbase >= L.n) break;                         // uniform
        const uint32_t i = cbase + threadIdx.x * VEC;
        float rv[4] = {0.f, 0.f, 0.f, 0.f}, wv[4] = {1.f, 1.f, 1.f, 1.f};
        if (i < L.n) {
            load_quad(rl, i, L.n, vec, rv);
            load_quad(wl, i, L.n, vec, wv);
        }
        uint32_t key[4];
        uint32_t packed = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            key[q] = score_key(rv[q], wv[q], eps);
            const bool valid = i + q < L.n;
            packed += (valid && key[q] > thr) ? 1u : 0u;
            packed += (valid && key[q] == thr) ? 0x10000u : 0u;
        }
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan(packed, slot[c & 1], &tot);
        uint32_t gpre = G + (ex & 0xffffu);
        uint32_t epre = E + (ex >> 16);
        if (packed) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (i + q >= L.n) break;
                if (key[q] > thr) {
                    const uint32_t pos = gpre + min(epre, quota);
                    if (pos < L.k) {             // always true for a threshold that belongs to this data
                        io[pos] = (uint32_t)(L.offset + i + q);
                        vo[pos] = rv[q];
                    }
                    ++gpre;
                } else if (key[q] == thr) {
                    const uint32_t pos = gpre + epre;
                    if (epre < quota && pos < L.k) {
                        io[pos] = (uint32_t)(L.offset + i + q);
                        vo[pos] = rv[q];
                    }
                    ++epre;
                }
            }
        }
        G += tot & 0xffffu;
        E += tot >> 16;
    }
}

// The importance keys themselves, for tests of the device arithmetic.
__global__ __launch_bounds__(BLOCK) void k_score_keys(const float* __restrict__ w, const float* __restrict__ r,
                                                      uint32_t n, float eps, uint32_t* __restrict__ key_out) {
    const uint64_t stride = (uint64_t)gridDim.x * BLOCK;
    for (uint64_t i = (uint64_t)blockIdx.x * BLOCK + threadIdx.x; i < n; i += stride) key_out[i] = score_key(r[i], w[i], eps);
}

// Plain 128-bit copy: the practical HBM ceiling every result is quoted against,
// and the known-size reference that scales the profiler's byte counters.
__global__ __launch_bounds__(BLOCK) void k_copy(float* __restrict__ dst, const float* __restrict__ src, uint64_t n) {
    const uint64_t quads = n / 4;
    const uint64_t stride = (uint64_t)gridDim.x * BLOCK;
    for (uint64_t q = (uint64_t)blockIdx.x * BLOCK + threadIdx.x; q < quads; q += stride)
        reinterpret_cast<float4*>(dst)[q] = reinterpret_cast<const float4*>(src)[q];
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) dst[quads * 4 + threadIdx.x] = src[quads * 4 + threadIdx.x];
}

}  // namespace iwp
