// Threshold mode: the front end exactly as Algorithm 1 prints it.  Each of the
// n_lead randomly chosen nodes of a layer marks the elements whose importance is
// strictly above the layer's threshold (mask line; fixed thresholds, Section 4.1),
// the masks are encoded one bit per element (encode_uint8: bit i%8 of byte i/8,
// i.e. bit i%32 of little-endian word i/32; a layer's mask is a whole number of
// words) and OR-ed, and every node splits its accumulated gradient by the common
// mask (G~ / G lines).  The number of sent elements is data dependent, so the
// layers' pairs are packed by a scan over device-resident counts.
//
// One look per chosen node (16 B/element), no selection at all; the other nodes
// stream once and hand over / clear their masked values on the way, with the
// 4096-bit tile mask taken straight from the encoded mask.
#pragma once

#include "iwp_common.hpp"

namespace iwp {

constexpr uint32_t MAX_LEAD = 8;                 // chosen nodes per layer

// The node in slot q of layer j (out-of-range entries read as node 0).
__device__ __forceinline__ uint32_t chosen_at(const uint32_t* __restrict__ leaders, uint32_t n_lead, uint32_t j,
                                              uint32_t q, uint32_t W) {
    const uint32_t l = leaders[(size_t)j * n_lead + q];
    return l < W ? l : 0u;
}

// Is node p among the first `upto` chosen nodes of layer j?
__device__ __forceinline__ bool chosen_before(const uint32_t* __restrict__ leaders, uint32_t n_lead, uint32_t j,
                                              uint32_t upto, uint32_t W, uint32_t p) {
    for (uint32_t q = 0; q < upto; ++q)
        if (chosen_at(leaders, n_lead, j, q, W) == p) return true;
    return false;
}

// Status words at the end of count_out: [n_layers] = total pairs, [n_layers + 1] = 1 if
// the total exceeds the caller's capacity (then nothing is exchanged).
__device__ __forceinline__ bool overflowed(const uint32_t* __restrict__ count_out, uint32_t n_layers) {
    return count_out[n_layers + 1] != 0u;
}

// Random gradient selection (Section 3.3): an element not above the threshold is still
// sent with probability importance / threshold.  The draw comes from Philox-4x32 with 10
// rounds (Salmon et al., SC'11): key = the caller's 64-bit seed, counter = (i / 4, layer,
// step low, step high); element i of the layer takes output word i % 4, and
// u = (word >> 8) * 2^-24.  It depends on (seed, step, layer, position) only, so every
// node, and any other implementation of the same generator, sees the same draw.
struct RandomSel {
    uint32_t on, key0, key1, step0, step1;
};

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// One tile of a chosen node in registers: residual (after adding the gradient and storing
// it back when gp is set) and weights, 16 values per lane; positions past the layer's end
// read as r = 0, w = 1.
__device__ __forceinline__ void chosen_tile(const float* gp, float* rl, const float* gl, const float* wl, float m,
                                            uint32_t n, uint32_t base, uint32_t tid, float (&rv)[CHUNKS_PER_TILE][4],
                                            float (&wv)[CHUNKS_PER_TILE][4]) {
    const bool vec = is_aligned16(rl) && is_aligned16(wl) && (!gp || is_aligned16(gl));
    if (vec && base + TILE <= n) {
        v4f rr[CHUNKS_PER_TILE], gg[CHUNKS_PER_TILE], ww[CHUNKS_PER_TILE];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            rr[u] = load_v4<true>(rl + i);
            if (gp) gg[u] = load_v4<true>(gl + i);
            ww[u] = load_v4<true>(wl + i);
        }
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
            if (gp) {
                rr[u] = accum(rr[u], gg[u], m);
                store_v4<true>(rl + i, rr[u]);
            }
            rv[u][0] = rr[u].x; rv[u][1] = rr[u].y; rv[u][2] = rr[u].z; rv[u][3] = rr[u].w;
            wv[u][0] = ww[u].x; wv[u][1] = ww[u].y; wv[u][2] = ww[u].z; wv[u][3] = ww[u].w;
        }
    } else {
        // ragged tail or misaligned base: the same shape, every load inside the layer issued before the first use
        float gv[CHUNKS_PER_TILE][4];
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t i = base + u * CHUNK + tid * VEC;
#pragma unroll
            for (int c = 0; c < 4; ++c) { rv[u][c] = 0.0f; wv[u][c] = 1.0f; }
            if (i < n) {
                load_quad<true>(rl, i, n, vec, rv[u]);
                if (gp) load_quad<true>(gl, i, n, vec, gv[u]);
                load_quad<true>(wl, i, n, vec, wv[u], 1.0f);
            }
        }
        if (gp) {
#pragma unroll
            for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
                const uint32_t i = base + u * CHUNK + tid * VEC;
                if (i < n) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) rv[u][c] = accum(rv[u][c], gv[u][c], m);
                    store_quad<true>(rl, i, n, vec, rv[u]);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Chosen nodes: accumulate (if asked), score, compare, encode.  Grid: n_lead * tiles.
// A node that appears in an earlier slot of the same layer is skipped (same mask).
// lmask: n_lead masks of mask_words words each, laid out like the final mask.
// thr: one value per layer, or per (layer, slot) with thr_per_slot.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_leader_mask(WorkerPtrs P, const float* __restrict__ w,
                                                       const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                       uint32_t tiles, const uint32_t* __restrict__ leaders,
                                                       uint32_t n_lead, uint32_t W, const float* __restrict__ thr,
                                                       bool thr_per_slot, bool accumulate, RandomSel rs, float eps,
                                                       uint32_t* __restrict__ lmask, uint64_t mask_words) {
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1);
    const uint32_t q = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - q * tiles;
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t p = chosen_at(leaders, n_lead, j, q, W);
    if (chosen_before(leaders, n_lead, j, q, W, p)) return;
    const uint32_t lt = t - L.tile_begin;
    const uint32_t base = lt * TILE;
    const float* gp = accumulate ? P.g[p] : nullptr;
    const float th = thr_per_slot ? thr[(size_t)j * n_lead + q] : thr[j];
    const uint32_t nwords = (L.n + 31) / 32;
    uint32_t* mw = lmask + (size_t)q * mask_words + L.mask_begin;
    float rv[CHUNKS_PER_TILE][4], wv[CHUNKS_PER_TILE][4];
    chosen_tile(gp, P.r[p] + L.offset, gp ? gp + L.offset : nullptr, w + L.offset, P.momentum, L.n, base, tid, rv, wv);
#pragma unroll
    for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
        const uint32_t i = base + u * CHUNK + tid * VEC;
        uint32_t nib = 0;
        uint32_t word4[4] = {0u, 0u, 0u, 0u};
        if (rs.on) philox4x32_10(i >> 2, j, rs.step0, rs.step1, rs.key0, rs.key1, word4);   // i is a multiple of 4
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float s = fabsf(rv[u][c]) / (fabsf(wv[u][c]) + eps);
            bool send = s > th;
            if (rs.on) {
                const float draw = (float)(word4[c] >> 8) * 0x1p-24f;
                const float prob = s / th;
                send = send || draw < prob;
            }
            if (i + c < L.n && send) nib |= 1u << c;
        }
        // eight lanes (32 consecutive elements) make one word of the encoded mask
        uint32_t word = nib << (4u * (lane & 7u));
        word |= __shfl_xor(word, 1, WAVE);
        word |= __shfl_xor(word, 2, WAVE);
        word |= __shfl_xor(word, 4, WAVE);
        const uint32_t widx = lt * TILE_WORDS + u * (CHUNK / 32) + (tid >> 3);
        if ((lane & 7u) == 0u && widx < nwords) mw[widx] = word;
    }
}

// ---------------------------------------------------------------------------
// Layer-wise threshold, part 1 (Section 3.4, Eq. 4): the chosen nodes accumulate and
// score, and every tile leaves the sum of its importance values and the sum of their
// squared deviations from the tile's own mean, both binary64.  Grid: n_lead * tiles.
// tile_stats[q * tiles + t] = (sum, squared deviations).
// ---------------------------------------------------------------------------
__device__ __forceinline__ double block_sum_f64(double v, double* slot) {
#pragma unroll
    for (int d = WAVE / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, WAVE);
    __syncthreads();                             // slot may still be read from an earlier call
    if ((threadIdx.x & (WAVE - 1)) == 0) slot[threadIdx.x >> 6] = v;
    __syncthreads();
    return ((slot[0] + slot[1]) + slot[2]) + slot[3];
}

__global__ __launch_bounds__(BLOCK) void k_leader_stats(WorkerPtrs P, const float* __restrict__ w,
                                                        const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                        uint32_t tiles, const uint32_t* __restrict__ leaders,
                                                        uint32_t n_lead, uint32_t W, float eps,
                                                        double2* __restrict__ tile_stats) {
    __shared__ double slot[BLOCK / WAVE];
    const uint32_t tid = threadIdx.x;
    const uint32_t q = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - q * tiles;
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t p = chosen_at(leaders, n_lead, j, q, W);
    if (chosen_before(leaders, n_lead, j, q, W, p)) return;
    const uint32_t base = (t - L.tile_begin) * TILE;
    const float* gp = P.g[p];
    float rv[CHUNKS_PER_TILE][4], wv[CHUNKS_PER_TILE][4];
    chosen_tile(gp, P.r[p] + L.offset, gp ? gp + L.offset : nullptr, w + L.offset, P.momentum, L.n, base, tid, rv, wv);
    float sc[CHUNKS_PER_TILE][4];
    double lane_sum = 0.0;
#pragma unroll
    for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
        const uint32_t i = base + u * CHUNK + tid * VEC;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            sc[u][c] = fabsf(rv[u][c]) / (fabsf(wv[u][c]) + eps);
            if (i + c < L.n) lane_sum += (double)sc[u][c];
        }
    }
    const double sum = block_sum_f64(lane_sum, slot);
    const double mean = sum / (double)min(TILE, L.n - base);
    double lane_m2 = 0.0;
#pragma unroll
    for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
        const uint32_t i = base + u * CHUNK + tid * VEC;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double d = (double)sc[u][c] - mean;
            if (i + c < L.n) lane_m2 += d * d;
        }
    }
    const double m2 = block_sum_f64(lane_m2, slot);
    if (tid == 0) tile_stats[(size_t)q * tiles + t] = make_double2(sum, m2);
}

// ---------------------------------------------------------------------------
// Layer-wise threshold, part 2: one workgroup per (layer, slot) merges the tiles
// (sum of squared deviations about the layer mean = sum over tiles of the tile's own
// plus n_t * (tile mean - layer mean)^2), then applies the rule:
// ratio = var / mean; thr = alpha + beta * ratio if ratio > C, else alpha - beta * ratio.
// stats_out[slot] = (mean, population variance), thr_out[slot] = thr rounded to binary32.
// A slot repeating an earlier node of the layer takes that node's tiles.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_layer_thr(const DevLayer* __restrict__ layers, uint32_t tiles,
                                                     const uint32_t* __restrict__ leaders, uint32_t n_lead, uint32_t W,
                                                     const double2* __restrict__ tile_stats, double alpha, double beta,
                                                     double C, double2* __restrict__ stats_out,
                                                     float* __restrict__ thr_out) {
    __shared__ double slot[BLOCK / WAVE];
    const uint32_t j = blockIdx.x / n_lead;
    const uint32_t q = blockIdx.x - j * n_lead;
    const DevLayer L = layers[j];
    const uint32_t p = chosen_at(leaders, n_lead, j, q, W);
    uint32_t q0 = 0;
    while (chosen_at(leaders, n_lead, j, q0, W) != p) ++q0;      // ends at q at the latest
    const uint32_t ntiles = (L.n + TILE - 1) / TILE;
    const double2* ts = tile_stats + (size_t)q0 * tiles + L.tile_begin;
    double part = 0.0;
    for (uint32_t t = threadIdx.x; t < ntiles; t += BLOCK) part += ts[t].x;
    const double n = (double)L.n;
    const double mean = L.n ? block_sum_f64(part, slot) / n : 0.0;
    part = 0.0;
    for (uint32_t t = threadIdx.x; t < ntiles; t += BLOCK) {
        const double nt = (double)min(TILE, L.n - t * TILE);
        const double d = ts[t].x / nt - mean;
        part += ts[t].y + nt * (d * d);
    }
    const double var = L.n ? block_sum_f64(part, slot) / n : 0.0;
    if (threadIdx.x == 0) {
        const double ratio = var / mean;
        const double thr = ratio > C ? alpha + beta * ratio : alpha - beta * ratio;
        stats_out[blockIdx.x] = make_double2(mean, var);
        thr_out[blockIdx.x] = (float)thr;
    }
}

// ---------------------------------------------------------------------------
// OR of the chosen nodes' masks -> the layer's mask (an output), and how many bits
// each tile holds.  One workgroup per super-tile, one wavefront per tile.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_mask_or_count(const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                         const uint32_t* __restrict__ leaders, uint32_t n_lead,
                                                         uint32_t W, const uint32_t* __restrict__ lmask,
                                                         uint64_t mask_words, uint32_t* __restrict__ mask_out,
                                                         uint2* __restrict__ tile_counts,
                                                         uint2* __restrict__ stile_counts) {
    __shared__ uint32_t cg[GROUP];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const uint32_t s = blockIdx.x;
    const uint32_t j = find_layer<true>(layers, n_layers, s);
    const DevLayer L = layers[j];
    const uint32_t ntiles = (L.n + TILE - 1) / TILE;
    const uint32_t nwords = (L.n + 31) / 32;
    const uint32_t lt0 = (s - L.stile_begin) * GROUP;
    const uint32_t nt = min(GROUP, ntiles - lt0);
    for (uint32_t tl = wave; tl < nt; tl += BLOCK / WAVE) {
        uint32_t c = 0;
#pragma unroll
        for (uint32_t h = 0; h < 2; ++h) {
            const uint32_t widx = (lt0 + tl) * TILE_WORDS + 2 * lane + h;
            if (widx < nwords) {
                uint32_t wd = 0;
                for (uint32_t q = 0; q < n_lead; ++q) {
                    const uint32_t p = chosen_at(leaders, n_lead, j, q, W);
                    if (!chosen_before(leaders, n_lead, j, q, W, p)) wd |= lmask[(size_t)q * mask_words + L.mask_begin + widx];
                }
                mask_out[L.mask_begin + widx] = wd;
                c += __popc(wd);
            }
        }
#pragma unroll
        for (int d = WAVE / 2; d > 0; d >>= 1) c += __shfl_xor(c, d, WAVE);
        if (lane == 0) cg[tl] = c;
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t G = 0;
        for (uint32_t tl = 0; tl < nt; ++tl) {
            tile_counts[L.tile_begin + lt0 + tl] = make_uint2(G, 0u);
            G += cg[tl];
        }
        stile_counts[s] = make_uint2(G, 0u);
    }
}

// ---------------------------------------------------------------------------
// Layer totals -> where each layer's pairs start in the packed outputs, the counts
// the caller sees, and the capacity check.  One workgroup.
// lay_out[j] = first pair of layer j, lay_out[n_layers] = total.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_layer_offsets(const uint32_t* __restrict__ layer_total, uint32_t n_layers,
                                                         uint32_t max_pairs, uint32_t* __restrict__ lay_out,
                                                         uint32_t* __restrict__ count_out) {
    __shared__ uint32_t slot[4];
    uint32_t carry = 0;
    for (uint32_t b = 0; b < n_layers; b += BLOCK) {
        const uint32_t j = b + threadIdx.x;
        const uint32_t v = j < n_layers ? layer_total[j] : 0u;
        uint32_t tot;
        const uint32_t ex = block_exclusive_scan(v, slot, &tot);
        if (j < n_layers) {
            lay_out[j] = carry + ex;
            count_out[j] = v;
        }
        carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        lay_out[n_layers] = carry;
        count_out[n_layers] = carry;
        count_out[n_layers + 1] = carry > max_pairs ? 1u : 0u;
    }
}

// ---------------------------------------------------------------------------
// The masked positions as ascending flat indices, layers packed in table order.
// One wavefront per tile; tile_out[t] = first pair of the tile inside its layer.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_mask_emit(const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                     uint32_t tiles_total, const uint32_t* __restrict__ mask,
                                                     const uint2* __restrict__ tile_counts,
                                                     const uint2* __restrict__ stile_counts,
                                                     const uint32_t* __restrict__ lay_out,
                                                     const uint32_t* __restrict__ count_out, uint32_t max_pairs,
                                                     uint32_t* __restrict__ tile_out, uint32_t* __restrict__ idx_out) {
    const uint32_t lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const uint32_t t = blockIdx.x * (BLOCK / WAVE) + wave;
    if (t >= tiles_total) return;
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const uint32_t lt = t - L.tile_begin;
    const uint32_t in_layer = stile_counts[L.stile_begin + lt / GROUP].x + tile_counts[t].x;
    if (lane == 0) tile_out[t] = in_layer;
    if (overflowed(count_out, n_layers)) return;
    const uint32_t nwords = (L.n + 31) / 32;
    uint32_t wd[2];
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
        const uint32_t widx = lt * TILE_WORDS + 2 * lane + h;
        wd[h] = widx < nwords ? mask[L.mask_begin + widx] : 0u;
    }
    const uint32_t c = __popc(wd[0]) + __popc(wd[1]);
    uint32_t pos = lay_out[j] + in_layer + wave_inclusive_scan(c) - c;
    const uint32_t first = (uint32_t)L.offset + lt * TILE + 2 * lane * 32;
#pragma unroll
    for (uint32_t h = 0; h < 2; ++h) {
        uint32_t m = wd[h];
        while (m) {
            const uint32_t b = __ffs(m) - 1;
            if (pos < max_pairs) idx_out[pos] = first + h * 32 + b;
            ++pos;
            m &= m - 1;
        }
    }
}

// ---------------------------------------------------------------------------
// Every node that is not chosen for the layer and has a gradient: accumulate, and
// where the tile's mask has bits, copy the accumulated value into the node's gather
// row and leave +0 behind.  Grid: W * tiles.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_follow_mask(WorkerPtrs P, const DevLayer* __restrict__ layers,
                                                       uint32_t n_layers, uint32_t tiles,
                                                       const uint32_t* __restrict__ leaders, uint32_t n_lead, uint32_t W,
                                                       const uint32_t* __restrict__ mask,
                                                       const uint32_t* __restrict__ tile_out,
                                                       const uint32_t* __restrict__ lay_out,
                                                       const uint32_t* __restrict__ count_out, uint32_t max_pairs,
                                                       float* __restrict__ gathered) {
    __shared__ uint32_t map[TILE_WORDS], pre[TILE_WORDS], slot[4];
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x / tiles;
    const uint32_t t = blockIdx.x - p * tiles;
    const uint32_t j = find_layer<false>(layers, n_layers, t);
    const DevLayer L = layers[j];
    const float* gp = P.g[p];
    if (!gp || chosen_before(leaders, n_lead, j, n_lead, W, p)) return;   // chosen / static nodes: pair by pair later
    const uint32_t lt = t - L.tile_begin;
    const uint32_t base = lt * TILE;
    float* rl = P.r[p] + L.offset;
    const float* gl = gp + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(gl);
    const bool full = vec && base + TILE <= L.n;
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
    const bool exchange = !overflowed(count_out, n_layers);
    const uint32_t nwords = (L.n + 31) / 32;
    if (tid < TILE_WORDS) {
        const uint32_t widx = lt * TILE_WORDS + tid;
        map[tid] = (exchange && widx < nwords) ? mask[L.mask_begin + widx] : 0u;
    }
    __syncthreads();
    bitmap_prefix(map, pre, slot);
    const uint64_t row = (uint64_t)lay_out[j] + tile_out[t];
    float* go = gathered + (size_t)p * max_pairs + min(row, (uint64_t)max_pairs);
    const uint32_t room = (uint32_t)((uint64_t)max_pairs - min(row, (uint64_t)max_pairs));
    if (full) {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t loc = u * CHUNK + tid * VEC;
#pragma unroll
            for (int q = 0; q < 4; ++q) rv[u][q] = accum(rv[u][q], gv[u][q], P.momentum);
            const uint32_t nib = (map[loc >> 5] >> (loc & 31u)) & 0xFu;
            if (nib) {
                uint32_t rank = bitmap_rank(map, pre, loc);
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if ((nib >> q) & 1u) { if (rank < room) go[rank] = rv[u][q]; ++rank; rv[u][q] = 0.0f; }
            }
            v4f out; out.x = rv[u][0]; out.y = rv[u][1]; out.z = rv[u][2]; out.w = rv[u][3];
            store_v4<true>(rl + base + loc, out);
        }
    } else {
#pragma unroll
        for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
            const uint32_t loc = u * CHUNK + tid * VEC;
            const uint32_t i = base + loc;
            if (i < L.n) {
                const uint32_t nib = (map[loc >> 5] >> (loc & 31u)) & 0xFu;
                uint32_t rank = nib ? bitmap_rank(map, pre, loc) : 0u;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    rv[u][q] = accum(rv[u][q], gv[u][q], P.momentum);
                    if ((nib >> q) & 1u) { if (rank < room) go[rank] = rv[u][q]; ++rank; rv[u][q] = 0.0f; }
                }
                store_quad<true>(rl, i, L.n, vec, rv[u]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Ordered sum over the W nodes and the weight update, for a pair count that lives
// on the device.  A node that streamed the pair's layer (k_follow_mask) left its
// value in its gather row; the others (chosen for the layer, or without a gradient)
// are read and cleared here, pair by pair.  Fixed grid, strided over the pairs.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_reduce_update_counted(WorkerPtrs P, const DevLayer* __restrict__ layers,
                                                                 uint32_t n_layers,
                                                                 const uint32_t* __restrict__ leaders, uint32_t n_lead,
                                                                 uint32_t W, const uint32_t* __restrict__ lay_out,
                                                                 const uint32_t* __restrict__ count_out,
                                                                 uint32_t max_pairs, const float* __restrict__ gathered,
                                                                 const uint32_t* __restrict__ idx,
                                                                 float* __restrict__ w, float scale,
                                                                 float* __restrict__ sum_out, uint64_t flat_end) {
    if (overflowed(count_out, n_layers)) return;
    const uint32_t total = min(count_out[n_layers], max_pairs);
    for (uint64_t jj64 = (uint64_t)blockIdx.x * BLOCK + threadIdx.x; jj64 < total; jj64 += (uint64_t)gridDim.x * BLOCK) {
        const uint32_t jj = (uint32_t)jj64;
        uint32_t lo = 0, hi = n_layers;              // layer of pair jj: last layer with lay_out <= jj
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (lay_out[mid] <= jj) lo = mid; else hi = mid;
        }
        uint32_t direct = 0;                         // bit p: node p did not stream this layer
        for (uint32_t p = 0; p < W; ++p)
            if (!P.g[p]) direct |= 1u << p;
        for (uint32_t q = 0; q < n_lead; ++q) direct |= 1u << chosen_at(leaders, n_lead, lo, q, W);
        const uint32_t i = idx[jj];
        const bool ok = i < flat_end;
        float acc = 0.0f;
        for (uint32_t p = 0; p < W; ++p) {
            float v;
            if ((direct >> p) & 1u) {
                v = ok ? P.r[p][i] : 0.0f;
                if (ok) P.r[p][i] = 0.0f;
            } else {
                v = gathered[(size_t)p * max_pairs + jj];
            }
            acc = p == 0 ? v : acc + v;
        }
        sum_out[jj] = acc;
        if (ok) {
            const float t = scale * acc;
            w[i] = w[i] + t;
        }
    }
}

}  // namespace iwp
