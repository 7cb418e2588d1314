// Kernels of the exact per-layer selection ("choose threshold" of Alg. 1 taken as
// the k-th largest importance) and of the ordered split into (index, value) pairs.
// All of them are segmented: one launch covers every layer of a layer table.
//
// The selection is an MSB-first radix select on the 31-bit importance key
// (digits of 12 + 10 + 9 bits).  Look 1 (iwp_stream.hpp) histograms the top digit
// of every element.  Look 2 (k_stage) reads the leader's residual and weights once
// more and copies out, per tile, the only elements that can still matter: those whose
// top digit is >= b1, the bin that holds rank k (above b1 all of them are kept, the
// threshold lies among those inside b1), and histograms the second digit of those
// inside b1.  Every tile owns a fixed slot in the staging arrays, so look 2 needs no
// cross-workgroup coordination at all.  With a threshold hint (say, last step's
// thresholds) look 1 already copies out everything from a bin slightly below the
// hinted one; if the new b1 is not below that bin the copies are complete and look 2
// only reads the slots, not the layer.  Everything after that works on the staged
// copies, a few percent of the layer: k_refine2 histograms the third digit, k_count /
// k_write place every kept element at its rank in index order.  A tile whose
// candidates do not fit its slot (heavy ties, e.g. a tile that is all zeros) is marked
// RAW and is simply re-read from r and w by the later passes.  Both routes are exact.
//
// The second and third digit picks have no launches of their own: a finished histogram is
// the same for every reader, so each workgroup of the consuming kernel redoes the pick of its
// layer in its prologue (k_refine2 the second, k_count the third), and one elected workgroup
// per layer records it.  Likewise
// k_write sums the counts of the layer's earlier super-tiles itself unless a layer has so
// many that a scan launch (k_scan) is cheaper.  Kernel boundaries are the only
// synchronisation between workgroups.
#pragma once

#include "iwp_common.hpp"

namespace iwp {


// ---------------------------------------------------------------------------
// Workspace initialisation with vector stores (a fill kernel rather than a memset
// node, so the call sequence can be graph-captured): histograms to zero, layer
// states reset; for the single-layer entry points also the one-row layer table.
//
// The first n_layers workgroups each reset one layer's state and decide from which bin
// look 1 copies candidates out (LayerState.stage_bin): from the caller's threshold hint if
// there is one; otherwise from a sample of the layer -- 16 to 256 evenly spaced runs of 256
// elements (the whole layer if it has no more), scored exactly as look 1 will score them,
// histogrammed in LDS, and the bin of the sample's rank k * (sample size / n) taken as the
// estimate.  Either way the guess only decides whether look 2 has to read the layer again;
// it never changes a result.  The other workgroups clear the histograms.
// ---------------------------------------------------------------------------
struct SampleSource {      // what the sample is taken from; on == 0: no sampling
    WorkerPtrs P;
    const float* w;
    const uint32_t* leader;
    uint32_t W;
    float eps;
    uint32_t on;
};

constexpr uint32_t SAMPLE_RUN = WAVE * VEC;        // 256 consecutive elements, one quad per lane
constexpr uint32_t SAMPLE_RUNS = 256;              // at most 65536 sampled elements per layer
constexpr uint32_t SAMPLE_RANK = 256;              // rank of the estimated threshold inside the sample, about

__device__ __forceinline__ uint32_t sample_stage_bin(const DevLayer& L, const float* gp, const float* rp,
                                                     const float* __restrict__ w, float eps, float m, uint32_t* lh,
                                                     uint32_t* sh) {
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const float* rl = rp + L.offset;
    const float* gl = gp ? gp + L.offset : nullptr;
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl) && (!gp || is_aligned16(gl));
    const uint32_t runs_total = (uint32_t)(((uint64_t)L.n + SAMPLE_RUN - 1) / SAMPLE_RUN);
    // enough runs for the sample's rank to be about SAMPLE_RANK (a relative error of a few percent in the
    // count, well inside the slack of one bin), at most SAMPLE_RUNS, at least 16
    const uint64_t want = ((uint64_t)SAMPLE_RANK * L.n / L.k + SAMPLE_RUN - 1) / SAMPLE_RUN;
    const uint32_t runs = min(runs_total, (uint32_t)min((uint64_t)SAMPLE_RUNS, max((uint64_t)16, want)));
    for (uint32_t b = tid; b < HIST0; b += BLOCK) lh[b] = 0u;
    __syncthreads();
    constexpr uint32_t PER_ROUND = 8;                // runs a wavefront has in flight
    for (uint32_t i0 = wave; i0 < runs; i0 += (BLOCK / WAVE) * PER_ROUND) {
        float rv[PER_ROUND][4], gv[PER_ROUND][4], wv[PER_ROUND][4];
        uint32_t e[PER_ROUND];
#pragma unroll
        for (uint32_t c = 0; c < PER_ROUND; ++c) {
            const uint32_t i = i0 + c * (BLOCK / WAVE);
            const uint64_t run = (uint64_t)i * runs_total / runs;
            const uint64_t pos = run * SAMPLE_RUN + lane * VEC;
            e[c] = (i < runs && pos < L.n) ? (uint32_t)pos : 0xFFFFFFFFu;
            if (e[c] != 0xFFFFFFFFu) {
                load_quad(rl, e[c], L.n, vec, rv[c]);
                if (gp) load_quad(gl, e[c], L.n, vec, gv[c]);
                load_quad(wl, e[c], L.n, vec, wv[c], 1.0f);
            }
        }
#pragma unroll
        for (uint32_t c = 0; c < PER_ROUND; ++c) {
            if (e[c] == 0xFFFFFFFFu) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (e[c] + q >= L.n) break;
                const float v = gp ? accum(rv[c][q], gv[c][q], m) : rv[c][q];
                atomicAdd(&lh[score_key(v, wv[c][q], eps) >> digit_shift(0)], 1u);
            }
        }
    }
    __syncthreads();
    // every run but the layer's last is full, and the last is only sampled when all are
    const uint64_t sampled = runs == runs_total ? (uint64_t)L.n : (uint64_t)runs * SAMPLE_RUN;
    const uint32_t ks = (uint32_t)max((uint64_t)1, ((uint64_t)L.k * sampled + L.n - 1) / L.n);
    uint32_t bin, k_rem;
    block_pick<(int)HIST0>(lh, ks, sh, &bin, &k_rem);
    return bin;
}

__global__ __launch_bounds__(BLOCK) void k_init(uint32_t* __restrict__ words, uint64_t n_words,
                                                LayerState* __restrict__ state, uint32_t n_layers,
                                                const iwp_threshold* __restrict__ hint,
                                                const DevLayer* __restrict__ layers,
                                                DevLayer* __restrict__ single_table, DevLayer row, DevLayer sentinel,
                                                SampleSource S) {
    __shared__ uint32_t lh[HIST0];
    __shared__ uint32_t sh[BLOCK + 2];
    if (blockIdx.x >= n_layers) {
        const uint64_t stride = (uint64_t)(gridDim.x - n_layers) * BLOCK;
        for (uint64_t i = (uint64_t)(blockIdx.x - n_layers) * BLOCK + threadIdx.x; i < n_words; i += stride) words[i] = 0u;
        if (single_table && blockIdx.x == n_layers && threadIdx.x == 0) {
            single_table[0] = row;
            single_table[1] = sentinel;
        }
        return;
    }
    const uint32_t j = blockIdx.x;
    const DevLayer L = single_table ? row : layers[j];       // the one-row table is only being written by this launch
    // one bin of slack below the hinted / estimated threshold bin (a bin is 1/16 octave); a threshold in
    // bin 0 or 1 (among zero scores): look 1 stages nothing
    uint32_t guess = 0;
    if (hint) {
        guess = (hint[j].key & 0x7fffffffu) >> digit_shift(0);
    } else if (S.on && L.k > 0 && L.n > 0) {                 // uniform over the workgroup
        const uint32_t p = leader_of(S.leader, j, S.W);
        guess = sample_stage_bin(L, S.P.g[p], S.P.r[p], S.w, S.eps, S.P.momentum, lh, sh);
    }
    if (threadIdx.x == 0) {
        LayerState st;
        st.b1 = 0; st.k_rem0 = 0; st.p22 = 0; st.k_rem1 = 0; st.thr = 0; st.n_eq_take = 0; st.prestaged = 0;
        st.stage_bin = guess >= 2u ? guess - 1u : NO_STAGE_BIN;
        state[j] = st;
    }
}

// ---------------------------------------------------------------------------
// First digit pick, one workgroup per layer: the bin b1 of the 4096-bin histogram that holds
// rank k, and whether look 1's copies (staged from a hinted bin) already cover it.  This pick
// keeps a launch of its own: its histogram is too large for every tile's workgroup to re-read,
// and a summary of it would have to be built with atomics on a handful of addresses that all
// workgroups of look 1 hit (measured: look 1 nearly twice as slow).  A layer whose look 1
// flushed into several copies has them added up here first.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_first_pick(const DevLayer* __restrict__ layers, uint32_t* __restrict__ hist,
                                                      LayerState* __restrict__ state) {
    __shared__ uint32_t sh[BLOCK + 2];
    const uint32_t j = blockIdx.x;
    const DevLayer L = layers[j];
    if (L.k == 0) return;
    uint32_t* h0 = layer_hist(hist, L, 0);
    if (L.h0_copies > 1) {
        // fold the copies into the first one (this workgroup is the layer's only reader and writer here)
        constexpr uint32_t PER = HIST0 / BLOCK;                  // 16 consecutive bins per thread
        constexpr uint32_t Q = PER / 4;
        uint4 acc[Q];
#pragma unroll
        for (uint32_t q = 0; q < Q; ++q) acc[q] = make_uint4(0u, 0u, 0u, 0u);
        // the copies come in powers of two: two at a time, or four at a time with all loads issued first
        const uint32_t step = L.h0_copies == 2 ? 2u : 4u;
        for (uint32_t c0 = 0; c0 < L.h0_copies; c0 += step) {
            uint4 v[4][Q];
#pragma unroll
            for (uint32_t c = 0; c < 4; ++c)
#pragma unroll
                for (uint32_t q = 0; q < Q; ++q)
                    v[c][q] = c < step ? reinterpret_cast<const uint4*>(h0 + (size_t)(c0 + c) * HIST0 + threadIdx.x * PER)[q]
                                       : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
            for (uint32_t c = 0; c < 4; ++c)
#pragma unroll
                for (uint32_t q = 0; q < Q; ++q) {
                    acc[q].x += v[c][q].x; acc[q].y += v[c][q].y; acc[q].z += v[c][q].z; acc[q].w += v[c][q].w;
                }
        }
        uint4* mine = reinterpret_cast<uint4*>(h0 + threadIdx.x * PER);
#pragma unroll
        for (uint32_t q = 0; q < Q; ++q) mine[q] = acc[q];
        __syncthreads();                                         // the pick below reads what the others stored
    }
    uint32_t bin, k_rem;
    block_pick<(int)HIST0>(h0, L.k, sh, &bin, &k_rem);
    if (threadIdx.x == 0) {
        const uint32_t stage_bin = state[j].stage_bin;
        state[j].b1 = bin;
        state[j].k_rem0 = k_rem;
        state[j].prestaged = (stage_bin != NO_STAGE_BIN && stage_bin <= bin) ? 1u : 0u;
    }
}

// ---------------------------------------------------------------------------
// Last digit pick on its own, one workgroup per layer, for the call that stops at the
// threshold (select_threshold): the exact k-th largest key and the number of ties to keep.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_final_pick(const DevLayer* __restrict__ layers, const uint32_t* __restrict__ hist,
                                                      LayerState* __restrict__ state, iwp_threshold* __restrict__ thr_out) {
    __shared__ uint32_t sh[BLOCK + 2];
    const uint32_t j = blockIdx.x;
    const DevLayer L = layers[j];
    if (L.k == 0) return;
    const uint32_t p22 = state[j].p22, k_rem1 = state[j].k_rem1;
    uint32_t bin, k_rem;
    block_pick<(int)HIST2>(layer_hist(hist, L, 2), k_rem1, sh, &bin, &k_rem);
    if (threadIdx.x == 0) {
        state[j].thr = (p22 << digit_bits(2)) | bin;
        state[j].n_eq_take = k_rem;
        if (thr_out) {
            iwp_threshold th;
            th.key = (p22 << digit_bits(2)) | bin; th.n_gt = L.k - k_rem; th.n_eq_take = k_rem;
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
    st.b1 = 0; st.k_rem0 = 0; st.p22 = 0; st.k_rem1 = 0;
    st.thr = thr[j].key; st.n_eq_take = thr[j].n_eq_take;
    st.stage_bin = NO_STAGE_BIN; st.prestaged = 0;
    state[j] = st;
}

// LDS histogram -> global, non-empty bins only.
template <int NB>
__device__ __forceinline__ void flush_hist(const uint32_t* lh, uint32_t* __restrict__ gh) {
    for (uint32_t b = threadIdx.x; b < NB; b += BLOCK) {
        const uint32_t v = lh[b];
        if (v) atomicAdd(&gh[b], v);
    }
}

// ---------------------------------------------------------------------------
// Look 2: the second digit's histogram of the elements inside b1, and staged candidates
// for the passes that follow.  The unit of work is a tile; a workgroup takes the tiles
// blockIdx.x, blockIdx.x + gridDim.x, ... (the grid is capped: a launch of hundreds of
// thousands of workgroups that mostly have nothing to do costs more than their work).
//  * Look 1 already filled the layer's slots from a bin <= b1 (threshold hint or sample):
//    only the slots are read, by the first tile's unit of every STAGE_GROUP tiles, into one
//    LDS histogram that is flushed once.  In the steady state of a training run the
//    threshold's bin holds about as many elements as are kept; that many single atomics per
//    tile, or one flush per tile, would queue up on the histogram's few cache lines.  A tile
//    whose candidates overflowed its slot in look 1 (RAW) is read again from r and w by its
//    own unit, as below; its new count carries the RESTAGED flag, so the reader of look-1
//    slots leaves it alone whether it sees the old or the new count.
//  * Otherwise the tile is read again from r and w: the elements whose top digit is >= b1
//    are copied into the tile's slot in index order (a tile with more candidates than its
//    slot holds is marked RAW), those inside b1 go into the histogram.
// ---------------------------------------------------------------------------
constexpr uint32_t STAGE_GROUP = 16;               // tiles whose slots one unit histograms
constexpr uint32_t STAGE_MAX_GRID = 32768;         // with at most 2^20 tiles per table: at most 32 tiles per workgroup
constexpr uint32_t STAGE_TILES_MAX = 64;           // ... and one per STAGE_TILES_PER_AVG tiles of the average layer beyond
constexpr uint32_t STAGE_TILES_PER_AVG = 4096;     // that, up to the 64 the kernel handles: every workgroup flushes into
                                                   // its layer's one second-digit histogram, and same-address atomics
                                                   // queue up (a 2^30-element layer: 15 000 flushes of up to 1024 bins)
constexpr uint32_t STAGE_TILES = 4;                // tiles per workgroup on tables whose layers average STAGE_LONG_LAYER_TILES
constexpr uint32_t STAGE_LONG_LAYER_TILES = 256;   // tiles or more: most tiles have nothing to do when look 1 staged the
                                                   // layer, and a workgroup that only finds that out still costs a launch
                                                   // slot and two dependent loads (AlexNet-shaped: 3 us per step less; on
                                                   // the ResNet-50-shaped set, whose hints miss more often, 8 us more)

__global__ __launch_bounds__(BLOCK) void k_stage(ResidualPtrs R, const float* __restrict__ w,
                                                 const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                 uint32_t tiles, const uint32_t* __restrict__ leader, uint32_t W,
                                                 float eps, const LayerState* __restrict__ state,
                                                 uint32_t* __restrict__ hist, uint32_t* __restrict__ stage_cnt,
                                                 StageArrays A) {
    __shared__ uint32_t lh[HIST1];
    __shared__ uint32_t slot[4];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    // the workgroup's tiles are consecutive (at most 64: the host sizes the grid accordingly); their counts
    // from look 1 are fetched in one go, and a layer's row and state only when the layer changes, so that a
    // tile with nothing to do costs no memory access at all
    const uint32_t per = (tiles + gridDim.x - 1) / gridDim.x;
    const uint32_t t0 = blockIdx.x * per, t1 = min(t0 + per, tiles);
    const uint32_t my_cnt = (t0 + lane < t1) ? stage_cnt[t0 + lane] : 0u;
    uint32_t cur_j = 0xFFFFFFFFu, b1 = 0;
    bool prestaged = false;
    bool filled = false;                                   // lh holds counts of layer cur_j that are not flushed yet:
                                                           // one flush per workgroup and layer, however many tiles
    DevLayer L;
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t j = find_layer<false>(layers, n_layers, t);
        if (j != cur_j) {
            if (filled) {
                __syncthreads();
                flush_hist<HIST1>(lh, layer_hist(hist, L, 1));
                filled = false;
            }
            L = layers[j];
            b1 = state[j].b1;
            prestaged = state[j].prestaged != 0;
            cur_j = j;
        }
        if (L.k == 0) continue;
        const uint32_t lt = t - L.tile_begin;
        const bool do_slots = prestaged && lt % STAGE_GROUP == 0;
        const bool raw = prestaged && __shfl(my_cnt, (int)(t - t0), WAVE) == RAW_TILE;
        if (prestaged && !do_slots && !raw) continue;      // uniform
        if (!filled) {
            __syncthreads();                               // a flush above has read lh
            for (uint32_t b = tid; b < HIST1; b += BLOCK) lh[b] = 0u;
            __syncthreads();
            filled = true;
        }

        if (do_slots) {
            // a wavefront takes every fourth tile of the group; the counts and the first 256 entries of all
            // its tiles are requested before any of them is used
            const uint32_t ntiles = (L.n + TILE - 1) / TILE;
            const uint32_t last = min(lt + STAGE_GROUP, ntiles);
            constexpr uint32_t MINE = STAGE_GROUP / (BLOCK / WAVE);
            uint32_t cnt[MINE];
            uint32_t key[MINE][4];
#pragma unroll
            for (uint32_t m = 0; m < MINE; ++m) {
                const uint32_t tt = lt + wave + m * (BLOCK / WAVE);
                cnt[m] = tt < last ? stage_cnt[L.tile_begin + tt] : 0u;
                if (cnt[m] & RESTAGED) cnt[m] = 0u;        // overflowed in look 1 (RAW, or already filled again by
                                                           // the tile's own unit, which also histograms it)
            }
#pragma unroll
            for (uint32_t m = 0; m < MINE; ++m) {
                const uint64_t sbb = L.slot_begin + (uint64_t)(lt + wave + m * (BLOCK / WAVE)) * L.slot_cap;
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    const uint32_t e = q * WAVE + lane;
                    key[m][q] = e < cnt[m] ? A.key[sbb + e] : NOT_AN_ELEMENT;
                }
            }
#pragma unroll
            for (uint32_t m = 0; m < MINE; ++m) {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q)
                    if (key[m][q] != NOT_AN_ELEMENT && (key[m][q] >> digit_shift(0)) == b1)
                        atomicAdd(&lh[(key[m][q] >> digit_shift(1)) & (HIST1 - 1)], 1u);
                const uint64_t sbb = L.slot_begin + (uint64_t)(lt + wave + m * (BLOCK / WAVE)) * L.slot_cap;
                for (uint32_t e = 4 * WAVE + lane; e < cnt[m]; e += WAVE) {    // fuller slots: the rest
                    const uint32_t k2 = A.key[sbb + e];
                    if ((k2 >> digit_shift(0)) == b1) atomicAdd(&lh[(k2 >> digit_shift(1)) & (HIST1 - 1)], 1u);
                }
            }
        }

        if (!prestaged || raw) {                           // uniform: this tile is read again
            const float* rl = R.r[leader_of(leader, j, W)] + L.offset;
            const float* wl = w + L.offset;
            const bool vec = is_aligned16(rl) && is_aligned16(wl);
            const uint32_t base = lt * TILE;
            uint32_t key[CHUNKS_PER_TILE][4];
            float val[CHUNKS_PER_TILE][4];
            float wgt[CHUNKS_PER_TILE][4];
            const bool full = vec && base + TILE <= L.n;
            if (full) {
#pragma unroll
                for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
                    const uint32_t i = base + u * CHUNK + tid * VEC;
                    const v4f a = load_v4<true>(rl + i);
                    const v4f b = load_v4<true>(wl + i);
                    val[u][0] = a.x; val[u][1] = a.y; val[u][2] = a.z; val[u][3] = a.w;
                    wgt[u][0] = b.x; wgt[u][1] = b.y; wgt[u][2] = b.z; wgt[u][3] = b.w;
                }
            } else {
#pragma unroll
                for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
                    const uint32_t i = base + u * CHUNK + tid * VEC;
                    if (i < L.n) {
                        load_quad(rl, i, L.n, vec, val[u]);
                        load_quad(wl, i, L.n, vec, wgt[u], 1.0f);
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q) { val[u][q] = 0.0f; wgt[u][q] = 1.0f; }
                    }
                }
            }
#pragma unroll
            for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
                const uint32_t i = base + u * CHUNK + tid * VEC;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (full || i + q < L.n) {
                        key[u][q] = score_key(val[u][q], wgt[u][q], eps);
                    } else {
                        key[u][q] = NOT_AN_ELEMENT;
                    }
                }
            }
            // a tile whose keys are all the same (typically a tile of zero residuals in a layer whose threshold is
            // zero, where everything ties) is recorded as such: one entry instead of an overflowing slot
            const uint32_t k0 = score_key(rl[base], wl[base], eps);            // the tile's first element
            bool same = true;
#pragma unroll
            for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) same = same && (key[u][q] == k0 || key[u][q] == NOT_AN_ELEMENT);
            const bool uniform_tile = __syncthreads_and(same ? 1 : 0) != 0;
            const uint64_t sb = L.slot_begin + (uint64_t)lt * L.slot_cap;
            if (uniform_tile) {
                if (tid == 0) {
                    if ((k0 >> digit_shift(0)) == b1)
                        atomicAdd(&lh[(k0 >> digit_shift(1)) & (HIST1 - 1)], min(TILE, L.n - base));
                    A.key[sb] = k0;
                    stage_cnt[t] = UNIFORM_TILE;
                }
            } else {
#pragma unroll
                for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (key[u][q] != NOT_AN_ELEMENT && (key[u][q] >> digit_shift(0)) == b1)
                            atomicAdd(&lh[(key[u][q] >> digit_shift(1)) & (HIST1 - 1)], 1u);
                const uint32_t cnt = stage_tile(key, val, base, b1, L.slot_cap, sb, A, slot);
                if (tid == 0) stage_cnt[t] = (prestaged && cnt != RAW_TILE) ? (cnt | RESTAGED) : cnt;
            }
        }
    }
    if (filled) {
        __syncthreads();
        flush_hist<HIST1>(lh, layer_hist(hist, L, 1));
    }
}

// ---------------------------------------------------------------------------
// Third digit: histogram over the elements whose first two digits match the prefix
// (the prologue's pick appended to b1), taken from the tile slots (or from r, w for RAW
// tiles).  One workgroup per super-tile.
// ---------------------------------------------------------------------------
constexpr uint32_t STILE_MAX_GRID = 8192;          // k_refine2 / k_count: beyond this many super-tiles a workgroup takes
                                                   // several consecutive ones (one pick, one flush for all of them)

__global__ __launch_bounds__(BLOCK) void k_refine2(ResidualPtrs R, const float* __restrict__ w,
                                                   const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                   uint32_t stiles, const uint32_t* __restrict__ leader, uint32_t W,
                                                   float eps, LayerState* __restrict__ state,
                                                   const uint32_t* __restrict__ stage_cnt, StageArrays A,
                                                   uint32_t* __restrict__ hist) {
    __shared__ uint32_t lh[HIST2];
    __shared__ uint32_t sh[BLOCK + 2];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    const uint32_t per = (stiles + gridDim.x - 1) / gridDim.x;
    const uint32_t s0 = blockIdx.x * per, s1 = min(s0 + per, stiles);
    uint32_t cur_j = 0xFFFFFFFFu, prefix = 0;
    bool filled = false;                                   // lh holds counts of layer cur_j
    DevLayer L;
    for (uint32_t s = s0; s < s1; ++s) {
        const uint32_t j = find_layer<true>(layers, n_layers, s);
        if (j != cur_j) {
            if (filled) {
                __syncthreads();
                flush_hist<HIST2>(lh, layer_hist(hist, L, 2));
                filled = false;
            }
            L = layers[j];
            cur_j = j;
            if (L.k == 0) continue;
            // second pick, redone by every workgroup of the layer, from the finished second-digit histogram
            uint32_t bin1, k_rem1;
            block_pick<(int)HIST1>(layer_hist(hist, L, 1), state[j].k_rem0, sh, &bin1, &k_rem1);
            prefix = (state[j].b1 << digit_bits(1)) | bin1;                   // 22 bits
            if (s == L.stile_begin && tid == 0) {
                state[j].p22 = prefix;
                state[j].k_rem1 = k_rem1;
            }
            __syncthreads();                               // the flush above has read lh
            for (uint32_t b = tid; b < HIST2; b += BLOCK) lh[b] = 0u;
            __syncthreads();
            filled = true;
        }
        if (L.k == 0) continue;
        const uint32_t ntiles = (L.n + TILE - 1) / TILE;
        const uint32_t lt0 = (s - L.stile_begin) * GROUP;
        const uint32_t nt = min(GROUP, ntiles - lt0);
        // the super-tile's eight counts, one per lane; a wavefront takes tiles wave and wave + 4, the counts
        // and the first 256 entries of both requested before any of them is used
        const uint32_t my_cnt = lane < nt ? staged_entries(stage_cnt[L.tile_begin + lt0 + lane]) : 0u;
        constexpr uint32_t MINE = GROUP / (BLOCK / WAVE);
        uint32_t cnt[MINE];
        uint32_t key[MINE][4];
#pragma unroll
        for (uint32_t m = 0; m < MINE; ++m) {
            const uint32_t tl = wave + m * (BLOCK / WAVE);
            cnt[m] = __shfl(my_cnt, (int)tl, WAVE);
            const uint64_t sb = L.slot_begin + (uint64_t)(lt0 + tl) * L.slot_cap;
            if (cnt[m] == UNIFORM_TILE) {                  // all keys of the tile are the slot's one entry
                const uint32_t k0 = A.key[sb];
                if (lane == 0 && (k0 >> digit_shift(1)) == prefix)
                    atomicAdd(&lh[k0 & (HIST2 - 1)], min(TILE, L.n - (lt0 + tl) * TILE));
                cnt[m] = 0u;
            }
            if (cnt[m] == RAW_TILE) cnt[m] = 0u;           // read again below
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                const uint32_t e = q * WAVE + lane;
                key[m][q] = e < cnt[m] ? A.key[sb + e] : NOT_AN_ELEMENT;
            }
        }
#pragma unroll
        for (uint32_t m = 0; m < MINE; ++m) {
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (key[m][q] != NOT_AN_ELEMENT && (key[m][q] >> digit_shift(1)) == prefix)
                    atomicAdd(&lh[key[m][q] & (HIST2 - 1)], 1u);
            const uint64_t sb = L.slot_begin + (uint64_t)(lt0 + wave + m * (BLOCK / WAVE)) * L.slot_cap;
            for (uint32_t e = 4 * WAVE + lane; e < cnt[m]; e += WAVE) {        // fuller slots: the rest
                const uint32_t k2 = A.key[sb + e];
                if ((k2 >> digit_shift(1)) == prefix) atomicAdd(&lh[k2 & (HIST2 - 1)], 1u);
            }
        }
        const uint64_t raw_tiles = __ballot(my_cnt == RAW_TILE) & 0xFFull;    // the same in every wavefront
        if (raw_tiles) {                                                       // uniform
            const float* rl = R.r[leader_of(leader, j, W)] + L.offset;
            const float* wl = w + L.offset;
            const bool vec = is_aligned16(rl) && is_aligned16(wl);
            for (uint32_t tl = 0; tl < nt; ++tl) {
                if (!((raw_tiles >> tl) & 1ull)) continue;
                for (uint32_t u = 0; u < CHUNKS_PER_TILE; ++u) {
                    const uint32_t i = (lt0 + tl) * TILE + u * CHUNK + tid * VEC;
                    if (i >= L.n) break;
                    float rv[4], wv[4];
                    load_quad(rl, i, L.n, vec, rv);
                    load_quad(wl, i, L.n, vec, wv, 1.0f);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t key2 = score_key(rv[q], wv[q], eps);
                        if (i + q < L.n && (key2 >> digit_shift(1)) == prefix) atomicAdd(&lh[key2 & (HIST2 - 1)], 1u);
                    }
                }
            }
        }
    }
    if (filled) {
        __syncthreads();
        flush_hist<HIST2>(lh, layer_hist(hist, L, 2));
    }
}

// ---------------------------------------------------------------------------
// Ordered split, part 1: per tile, how many elements lie above the threshold and
// how many tie with it.  One workgroup per super-tile; writes each tile's exclusive
// prefix inside the super-tile and the super-tile's totals.  The threshold is the
// prologue's third pick (recorded, with thr_out, by the layer's first workgroup), or with
// FROM_RECORDS the caller's record (compact_pairs): then there is no stage table and
// every tile is re-read.
// ---------------------------------------------------------------------------
template <bool FROM_RECORDS>
__global__ __launch_bounds__(BLOCK) void k_count(ResidualPtrs R, const float* __restrict__ w,
                                                 const DevLayer* __restrict__ layers, uint32_t n_layers, uint32_t stiles,
                                                 const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                 LayerState* __restrict__ state, const uint32_t* __restrict__ hist,
                                                 iwp_threshold* __restrict__ thr_out,
                                                 const uint32_t* __restrict__ stage_cnt, StageArrays A,
                                                 uint2* __restrict__ tile_counts, uint2* __restrict__ stile_counts) {
    __shared__ uint32_t cg[GROUP], ce[GROUP];
    __shared__ uint32_t sh[BLOCK + 2];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & (WAVE - 1), wave = tid >> 6;
    constexpr bool all_raw = FROM_RECORDS;
    const uint32_t per = (stiles + gridDim.x - 1) / gridDim.x;
    const uint32_t s0 = blockIdx.x * per, s1 = min(s0 + per, stiles);
    uint32_t cur_j = 0xFFFFFFFFu, thr = 0;
    DevLayer L;
    for (uint32_t s = s0; s < s1; ++s) {
        const uint32_t j = find_layer<true>(layers, n_layers, s);
        if (j != cur_j) {
            L = layers[j];
            cur_j = j;
            if (L.k == 0) continue;
            if (FROM_RECORDS) {
                thr = state[j].thr;
            } else {
                // third pick, redone by every workgroup of the layer: the exact k-th largest key
                uint32_t bin2, k_rem2;
                block_pick<(int)HIST2>(layer_hist(hist, L, 2), state[j].k_rem1, sh, &bin2, &k_rem2);
                thr = (state[j].p22 << digit_bits(2)) | bin2;
                if (s == L.stile_begin && tid == 0) {
                    state[j].thr = thr;
                    state[j].n_eq_take = k_rem2;
                    if (thr_out) {
                        iwp_threshold th;
                        th.key = thr; th.n_gt = L.k - k_rem2; th.n_eq_take = k_rem2;
                        thr_out[j] = th;
                    }
                }
            }
        }
        if (L.k == 0) continue;
        const uint32_t ntiles = (L.n + TILE - 1) / TILE;
        const uint32_t lt0 = (s - L.stile_begin) * GROUP;       // first tile of the super-tile, in the layer
        const uint32_t nt = min(GROUP, ntiles - lt0);
        const float* rl = R.r[leader_of(leader, j, W)] + L.offset;
        const float* wl = w + L.offset;
        // each wavefront takes tiles of its own (tiles wave and wave + 4; the counts and the first 256 entries of
        // both requested before any of them is used); nothing workgroup-wide until the end
        const uint32_t my_cnt = (!all_raw && lane < nt) ? staged_entries(stage_cnt[L.tile_begin + lt0 + lane]) : RAW_TILE;
        constexpr uint32_t MINE = GROUP / (BLOCK / WAVE);
        uint32_t cnt[MINE];
        uint32_t key[MINE][4];
#pragma unroll
        for (uint32_t m = 0; m < MINE; ++m) {
            const uint32_t tl = wave + m * (BLOCK / WAVE);
            cnt[m] = __shfl(my_cnt, (int)tl, WAVE);
            const uint64_t sb = L.slot_begin + (uint64_t)(lt0 + tl) * L.slot_cap;
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                const uint32_t e = q * WAVE + lane;
                key[m][q] = (tl < nt && cnt[m] < UNIFORM_TILE && e < cnt[m]) ? A.key[sb + e] : NOT_AN_ELEMENT;
            }
        }
#pragma unroll
        for (uint32_t m = 0; m < MINE; ++m) {
            const uint32_t tl = wave + m * (BLOCK / WAVE);
            if (tl >= nt) continue;
            uint32_t gt = 0, eq = 0;
            if (cnt[m] == UNIFORM_TILE) {                  // all keys of the tile are the slot's one entry
                const uint32_t k0 = A.key[L.slot_begin + (uint64_t)(lt0 + tl) * L.slot_cap];
                const uint32_t n_tile = min(TILE, L.n - (lt0 + tl) * TILE);
                if (lane == 0) { gt = k0 > thr ? n_tile : 0u; eq = k0 == thr ? n_tile : 0u; }
            } else if (cnt[m] != RAW_TILE) {
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    gt += (key[m][q] != NOT_AN_ELEMENT && key[m][q] > thr) ? 1u : 0u;
                    eq += key[m][q] == thr ? 1u : 0u;          // a key is never NOT_AN_ELEMENT (bit 31 is clear)
                }
                const uint64_t sb = L.slot_begin + (uint64_t)(lt0 + tl) * L.slot_cap;
                for (uint32_t e = 4 * WAVE + lane; e < cnt[m]; e += WAVE) {
                    const uint32_t k2 = A.key[sb + e];
                    gt += k2 > thr ? 1u : 0u;
                    eq += k2 == thr ? 1u : 0u;
                }
            } else {
                const uint32_t first = (lt0 + tl) * TILE;
                const uint32_t end = min(L.n, first + TILE);
                for (uint32_t i = first + lane; i < end; i += WAVE) {
                    const uint32_t k2 = score_key(rl[i], wl[i], eps);
                    gt += k2 > thr ? 1u : 0u;
                    eq += k2 == thr ? 1u : 0u;
                }
            }
#pragma unroll
            for (int d = WAVE / 2; d > 0; d >>= 1) {
                gt += __shfl_xor(gt, d, WAVE);
                eq += __shfl_xor(eq, d, WAVE);
            }
            if (lane == 0) { cg[tl] = gt; ce[tl] = eq; }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t G = 0, E = 0;
            for (uint32_t tl = 0; tl < nt; ++tl) {
                tile_counts[L.tile_begin + lt0 + tl] = make_uint2(G, E);
                G += cg[tl];
                E += ce[tl];
            }
            stile_counts[s] = make_uint2(G, E);
        }
        __syncthreads();                                        // cg / ce are written again for the next super-tile
    }
}

// Part 2: exclusive prefix of the super-tile totals inside each layer, in order.
// One workgroup per layer, eight consecutive super-tiles per lane and round.
// every_layer: also layers with k == 0 (threshold mode has no k); layer_total (may be
// NULL) receives the layer's first sum.
__global__ __launch_bounds__(BLOCK) void k_scan(const DevLayer* __restrict__ layers, uint2* __restrict__ stile_counts,
                                                bool every_layer, uint32_t* __restrict__ layer_total) {
    constexpr uint32_t PER = 8;
    __shared__ uint32_t slot_g[4], slot_e[4];
    const uint32_t j = blockIdx.x;
    if (layers[j].k == 0 && !every_layer) return;
    const uint32_t sb = layers[j].stile_begin;
    const uint32_t se = sb + (layers[j].n + STILE - 1) / STILE;
    uint32_t G = 0, E = 0;
    for (uint32_t b = sb; b < se; b += BLOCK * PER) {
        const uint32_t s0 = b + threadIdx.x * PER;
        uint2 v[PER];
        uint32_t lg = 0, le = 0;
#pragma unroll
        for (uint32_t q = 0; q < PER; ++q) {
            v[q] = (s0 + q < se) ? stile_counts[s0 + q] : make_uint2(0u, 0u);
            lg += v[q].x;
            le += v[q].y;
        }
        uint32_t tot_g, tot_e;
        uint32_t pg = G + block_exclusive_scan(lg, slot_g, &tot_g);
        uint32_t pe = E + block_exclusive_scan(le, slot_e, &tot_e);
#pragma unroll
        for (uint32_t q = 0; q < PER; ++q) {
            if (s0 + q < se) stile_counts[s0 + q] = make_uint2(pg, pe);
            pg += v[q].x;
            pe += v[q].y;
        }
        G += tot_g;
        E += tot_e;
        __syncthreads();
    }
    if (layer_total && threadIdx.x == 0) layer_total[j] = G;
}

// Part 3: write the pairs.  An element above the threshold goes to position
// (#above before it) + min(#ties before it, quota); a tie is kept iff fewer than
// `quota` ties precede it.  Positions are counted in index order, so the output is
// ascending and ties go to the lowest indices (Alg. 1 split: the sent part is the
// residual itself).  tile_out[t] receives the position of the tile's first pair.
// FUSED (whole-step entry point): the value also goes into the leader's row of the
// gather matrix and the leader's residual is cleared at the sent position.
// One wavefront per tile, four tiles (half a super-tile) per workgroup.  FOLD: the super-tile
// totals are as k_count left them and the workgroup adds up the layer's earlier ones itself;
// otherwise k_scan has turned them into prefixes.
template <bool FUSED, bool FOLD>
__global__ __launch_bounds__(BLOCK) void k_write(ResidualPtrs R, const float* __restrict__ w,
                                                 const DevLayer* __restrict__ layers, uint32_t n_layers,
                                                 const uint32_t* __restrict__ leader, uint32_t W, float eps,
                                                 const LayerState* __restrict__ state,
                                                 const uint32_t* __restrict__ stage_cnt, StageArrays A, bool all_raw,
                                                 const uint2* __restrict__ tile_counts,
                                                 const uint2* __restrict__ stile_counts,
                                                 uint32_t* __restrict__ tile_out,
                                                 uint32_t* __restrict__ idx_out, float* __restrict__ val_out,
                                                 float* __restrict__ gathered, uint64_t K) {
    __shared__ uint32_t maps[BLOCK / WAVE][4][TILE_WORDS];
    __shared__ uint32_t red[2][BLOCK / WAVE];
    const uint32_t lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x >> 6;
    const uint32_t s = blockIdx.x / (GROUP / (BLOCK / WAVE));            // the workgroup's super-tile
    const uint32_t part = blockIdx.x % (GROUP / (BLOCK / WAVE));
    const uint32_t j = find_layer<true>(layers, n_layers, s);
    const DevLayer L = layers[j];
    if (L.k == 0) return;
    const uint32_t ntiles = (L.n + TILE - 1) / TILE;
    const uint32_t lt = (s - L.stile_begin) * GROUP + part * (BLOCK / WAVE) + wave;
    if (lt - wave >= ntiles) return;                                      // uniform: nothing of this part exists
    uint2 sc;
    if (FOLD) {
        // elements above / tying in the layer's earlier super-tiles: summed here, by everybody
        uint32_t g = 0, e = 0;
        for (uint32_t q = L.stile_begin + threadIdx.x; q < s; q += BLOCK) {
            const uint2 c = stile_counts[q];
            g += c.x;
            e += c.y;
        }
#pragma unroll
        for (int d = WAVE / 2; d > 0; d >>= 1) {
            g += __shfl_xor(g, d, WAVE);
            e += __shfl_xor(e, d, WAVE);
        }
        if (lane == 0) { red[0][wave] = g; red[1][wave] = e; }
        __syncthreads();
        sc.x = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        sc.y = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    } else {
        sc = stile_counts[s];                                             // already scanned (k_scan)
    }
    if (lt >= ntiles) return;
    const uint32_t t = L.tile_begin + lt;
    const LayerState st = state[j];
    const uint32_t thr = st.thr, quota = st.n_eq_take;
    const uint32_t lead = leader_of(leader, j, W);
    float* rl = R.r[lead] + L.offset;
    const uint2 tc = tile_counts[t];
    const uint32_t Gt = sc.x + tc.x, Et = sc.y + tc.y;         // elements above / tying, before this tile
    const uint32_t out_base = Gt + min(Et, quota);
    const uint32_t tile_first = lt * TILE;
    uint32_t* io = idx_out + L.out_offset;
    float* vo = val_out + L.out_offset;
    float* go = FUSED ? gathered + (size_t)lead * K + L.out_offset : nullptr;
    if (lane == 0) tile_out[t] = out_base;
    const uint32_t cnt = all_raw ? RAW_TILE : staged_entries(stage_cnt[t]);

    if (cnt == UNIFORM_TILE) {
        // all keys of the tile are the slot's one entry: above the threshold everything is kept, at the
        // threshold the first elements until the quota of ties is used up, below it nothing
        const uint32_t k0 = A.key[L.slot_begin + (uint64_t)lt * L.slot_cap];
        const uint32_t n_tile = min(TILE, L.n - tile_first);
        uint32_t take = 0;
        if (k0 > thr) take = n_tile;
        else if (k0 == thr && Et < quota) take = min(n_tile, quota - Et);
        for (uint32_t i = lane; i < take; i += WAVE) {
            const uint32_t pos = out_base + i;
            const uint32_t li = tile_first + i;
            if (pos < L.k) {
                const float v = rl[li];
                io[pos] = (uint32_t)(L.offset + li);
                vo[pos] = v;
                if (FUSED) { go[pos] = v; rl[li] = 0.0f; }
            }
        }
        return;
    }
    if (cnt != RAW_TILE) {
        if (cnt == 0) return;
        uint32_t* eqmap = maps[wave][0];
        uint32_t* eqpre = maps[wave][1];
        uint32_t* selmap = maps[wave][2];
        uint32_t* selpre = maps[wave][3];
        const uint64_t sb = L.slot_begin + (uint64_t)lt * L.slot_cap;
        eqmap[2 * lane] = 0u; eqmap[2 * lane + 1] = 0u;
        selmap[2 * lane] = 0u; selmap[2 * lane + 1] = 0u;
        // a lane keeps up to PER of the tile's entries in registers (enough for the usual tile); the
        // rare fuller slot takes more rounds of the same three passes
        constexpr uint32_t PER = 2;
        for (uint32_t e0 = 0; e0 < cnt; e0 += PER * WAVE) {
            uint32_t key[PER], loc[PER];
            float val[PER];
            bool have[PER];
#pragma unroll
            for (uint32_t q = 0; q < PER; ++q) {
                const uint32_t e = e0 + q * WAVE + lane;
                have[q] = e < cnt;
                key[q] = have[q] ? A.key[sb + e] : 0u;
                loc[q] = have[q] ? (A.idx[sb + e] - tile_first) & (TILE - 1) : 0u;
                val[q] = have[q] ? A.val[sb + e] : 0.0f;
            }
            if (e0 == 0) {
                // ties first: all of the slot's entries equal to the threshold, in index order
                wave_sync();
                for (uint32_t e = lane; e < cnt; e += WAVE) {
                    if (e < PER * WAVE) continue;                         // those are in registers (below)
                    if (A.key[sb + e] == thr) {
                        const uint32_t l2 = (A.idx[sb + e] - tile_first) & (TILE - 1);
                        atomicOr(&eqmap[l2 >> 5], 1u << (l2 & 31u));
                    }
                }
#pragma unroll
                for (uint32_t q = 0; q < PER; ++q)
                    if (have[q] && key[q] == thr) atomicOr(&eqmap[loc[q] >> 5], 1u << (loc[q] & 31u));
                wave_sync();
                wave_bitmap_prefix(eqmap, eqpre);
                // then everything that is kept
                for (uint32_t e = lane; e < cnt; e += WAVE) {
                    if (e < PER * WAVE) continue;
                    const uint32_t k2 = A.key[sb + e];
                    const uint32_t l2 = (A.idx[sb + e] - tile_first) & (TILE - 1);
                    if (k2 > thr || (k2 == thr && Et + bitmap_rank(eqmap, eqpre, l2) < quota))
                        atomicOr(&selmap[l2 >> 5], 1u << (l2 & 31u));
                }
#pragma unroll
                for (uint32_t q = 0; q < PER; ++q)
                    if (have[q] && (key[q] > thr || (key[q] == thr && Et + bitmap_rank(eqmap, eqpre, loc[q]) < quota)))
                        atomicOr(&selmap[loc[q] >> 5], 1u << (loc[q] & 31u));
                wave_sync();
                wave_bitmap_prefix(selmap, selpre);
            }
#pragma unroll
            for (uint32_t q = 0; q < PER; ++q) {
                if (have[q] && ((selmap[loc[q] >> 5] >> (loc[q] & 31u)) & 1u)) {
                    const uint32_t pos = out_base + bitmap_rank(selmap, selpre, loc[q]);
                    const uint32_t li = tile_first + loc[q];
                    if (pos < L.k && li < L.n) {
                        io[pos] = (uint32_t)(L.offset + li);
                        vo[pos] = val[q];
                        if (FUSED) { go[pos] = val[q]; rl[li] = 0.0f; }
                    }
                }
            }
        }
        return;
    }

    // RAW tile: every element is scored again, 256 at a time
    const float* wl = w + L.offset;
    const bool vec = is_aligned16(rl) && is_aligned16(wl);
    uint32_t G = Gt, E = Et;
    for (uint32_t c = 0; c < TILE / (WAVE * VEC); ++c) {
        const uint32_t cbase = tile_first + c * (WAVE * VEC);
        if (cbase >= L.n) break;
        const uint32_t i = cbase + lane * VEC;
        float rv[4] = {0.f, 0.f, 0.f, 0.f}, wv[4] = {1.f, 1.f, 1.f, 1.f};
        if (i < L.n) {
            load_quad(rl, i, L.n, vec, rv);
            load_quad(wl, i, L.n, vec, wv, 1.0f);
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
        const uint32_t inc = wave_inclusive_scan(packed);
        const uint32_t tot = __shfl(inc, WAVE - 1, WAVE);
        const uint32_t ex = inc - packed;
        uint32_t gpre = G + (ex & 0xffffu);
        uint32_t epre = E + (ex >> 16);
        if (packed) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (i + q >= L.n) break;
                uint32_t pos = 0xFFFFFFFFu;
                if (key[q] > thr) { pos = gpre + min(epre, quota); ++gpre; }
                else if (key[q] == thr) { if (epre < quota) pos = gpre + epre; ++epre; }
                if (pos < L.k) {
                    io[pos] = (uint32_t)(L.offset + i + q);
                    vo[pos] = rv[q];
                    if (FUSED) { go[pos] = rv[q]; rl[i + q] = 0.0f; }
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

// Plain 128-bit copy, one quad per lane: the practical HBM ceiling every result is
// quoted against, and the known-size reference that scales the profiler's byte
// counters.
__global__ __launch_bounds__(BLOCK) void k_copy(float* __restrict__ dst, const float* __restrict__ src, uint64_t n) {
    const uint64_t quads = n / 4;
    const uint64_t q = (uint64_t)blockIdx.x * BLOCK + threadIdx.x;
    if (q < quads) reinterpret_cast<v4f*>(dst)[q] = reinterpret_cast<const v4f*>(src)[q];
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) dst[quads * 4 + threadIdx.x] = src[quads * 4 + threadIdx.x];
}

}  // namespace iwp
