// Oracle for the importance-weighted-pruning compression step (arXiv 1901.01544).
//
// TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded CPU
// definition of what the GPU path must compute.  It shares no code, header,
// table or helper with the HIP library and is called only by the tests, by the
// smoke check and by the benchmark's cpu_baseline leg.  The product path never
// routes through it.
//
// What it computes (paper, Algorithm 1, the body of the per-layer loop and the
// reduce/update lines after it; Section 3.2 for the importance measure):
//
//   O1  local accumulation      r[i] <- r[i] + g[i]                   (Alg. 1, the
//       accumulation line before the layer loop, read as residual accumulation;
//       Eq. 3 and the "for local accumulation" line)
//   O2  importance              s[i] = |r[i]| / (|w[i]| + eps)        (Alg. 1, mask line;
//       abstract: ratio of gradient to parameter value)
//   O3  selection               the k elements that come first under the total
//       order (score descending, index ascending): a full sort.  Stands in for
//       "choose threshold" + "Mask <- importance > thr" of Alg. 1 with the
//       threshold placed at the k-th largest score.
//   O4  split                   idx = selected positions ascending,
//       val[j] = r[idx[j]] bit for bit                                (Alg. 1, G~ = grad (.) Mask)
//   O5  reduce                  sum[j] = ((R_0[idx_j] + R_1[idx_j]) + ...) + R_{W-1}[idx_j]
//       fixed left fold starting from R_0's value                     (Alg. 1, ring all-reduce line)
//   O6  update                  w[idx_j] <- w[idx_j] + (scale * sum[j]), two roundings
//                                                                     (Alg. 1, SGD line; Eq. 3)
//   O7  clear                   R_p[idx_j] <- +0.0f for every worker  (Alg. 1, G = grad (.) not Mask)
//
// Arithmetic is IEEE-754 binary32, round to nearest even, denormals kept, no
// contraction (build with -ffp-contract=off, never -ffast-math).
//
// Threshold mode, the front end exactly as Algorithm 1 prints it (fixed thresholds
// of Section 4.1 instead of a k-th largest score):
//   T1  mask of one chosen node    m[i] = (s[i] > thr), strict           (Alg. 1, mask line)
//   T2  encoding                   bit i%8 of byte i/8, LSB first; one layer's mask is a
//       whole number of 32-bit words                                     (Alg. 1, encode_uint8 -- the paper
//       does not give the format; this is the build's reading)
//   T3  union over the chosen nodes  Mask = OR_i m_{r_i}                 (Alg. 1, OR line)
//   T4  split on EVERY node        sent: R_p[i] for Mask[i], kept: the rest   (Alg. 1, G~ / G lines)
//   then O5..O7 over the masked positions.
//
// Layer-wise threshold (Section 3.4, Eq. 4): the threshold of T1 is not given but derived,
// per layer and per chosen node, from that node's importance values:
//   L1  mean = (1/n) sum s[i],  var = (1/n) sum (s[i] - mean)^2  (population variance; the paper
//       says only "mean and variance"), two passes in binary64 over the binary32 scores
//   L2  ratio = var / mean;  thr = alpha + beta * ratio  if ratio > C,  else  alpha - beta * ratio
//       (Eq. 4 prints the same condition on both branches; the prose after it raises the
//       threshold for a large ratio and lowers it otherwise), binary64, rounded once to binary32
//   then T1..T4 with each chosen node using its own threshold.
//
// Momentum-weighted residual (Eq. 3: what is sparsified is m * g_{t-1} + g_t, the residual
// "accumulated local with momentum"):
//   M1  r[i] <- (m * r[i]) + g[i], product rounded, then sum rounded (no contraction);
//       m = 1 is O1.  The whole-step functions take m and use M1 in place of O1.
//
// Random gradient selection (Section 3.3): an element that is not above the threshold is
// still sent with probability importance / threshold.
//   S1  the draw: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random
//       numbers: as easy as 1, 2, 3", SC'11), key = the 64-bit seed, counter = (i / 4, layer,
//       step low word, step high word); element i takes output word i % 4 and
//       u = (word >> 8) * 2^-24, a multiple of 2^-24 in [0, 1).  The draw depends on
//       (seed, step, layer, position) only, not on the node.
//   S2  p = s / thr in binary32;  m[i] = (s > thr) or (u < p).
//
// Pins (tests/test_oracle_pins.py): brute-force rank count on tiny layers,
// cardinality, exact conservation, the paper's 64x / 58.8x ratios as keep
// fractions, numpy lexsort cross-check, threshold-mask equivalence with the
// paper's "importance > thr" mask, dense masked formulation of the reduce and
// update, closed forms, exact-rational check of the divide, hand-worked example.
// No function here is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

extern "C" {

typedef struct {
    uint32_t key;        // bit pattern of the k-th largest score
    uint32_t n_gt;       // number of elements with score strictly above it
    uint32_t n_eq_take;  // how many of the elements equal to it are kept (lowest indices)
} oracle_threshold;

typedef struct {
    int64_t offset;       // first element of the layer in the flat buffers
    uint32_t n;           // elements in the layer
    uint32_t k;           // elements kept (0 = accumulate only)
    uint32_t out_offset;  // first pair of the layer in idx/val
    uint32_t pad;
} oracle_layer;


}  // extern "C"

namespace {

// Order-preserving integer image of a non-negative float: for s >= +0 the
// unsigned order of the bit patterns equals the float order; +inf sits above
// every finite value and a NaN (sign cleared) above +inf.
inline uint32_t score_key(float s) {
    uint32_t b;
    std::memcpy(&b, &s, sizeof b);
    return b & 0x7fffffffu;
}

struct Ranked {
    uint32_t key;
    uint32_t idx;
};

}  // namespace

extern "C" {

// O1.  Alg. 1 accumulation line / Eq. 3: one fp32 add per element.
void oracle_accumulate(float* r, const float* g, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) r[i] = r[i] + g[i];
}

// M1: local accumulation with momentum, r <- (m * r) + g, two roundings.
void oracle_accumulate_momentum(float* r, const float* g, uint64_t n, float m) {
    for (uint64_t i = 0; i < n; ++i) {
        float decayed = m * r[i];
        r[i] = decayed + g[i];
    }
}

// O2.  Alg. 1 mask line: importance of every element, eps added to |w| in fp32
// before the divide.
void oracle_score(const float* w, const float* r, uint64_t n, float eps, float* s) {
    for (uint64_t i = 0; i < n; ++i) {
        float denom = std::fabs(w[i]) + eps;
        s[i] = std::fabs(r[i]) / denom;
    }
}

// Integer keys of the scores (used by tests that want to look at the order).
void oracle_score_keys(const float* w, const float* r, uint64_t n, float eps, uint32_t* key) {
    for (uint64_t i = 0; i < n; ++i) {
        float denom = std::fabs(w[i]) + eps;
        key[i] = score_key(std::fabs(r[i]) / denom);
    }
}

// O3 + the index half of O4.  Full sort by (score descending, index ascending),
// keep the first k, return their positions in ascending order and the threshold
// record.  Returns 0, or -1 on k > n.
int oracle_select(const float* s, uint32_t n, uint32_t k, uint32_t* idx_out, oracle_threshold* thr) {
    if (k > n) return -1;
    if (thr) { thr->key = 0; thr->n_gt = 0; thr->n_eq_take = 0; }
    if (k == 0) return 0;
    std::vector<Ranked> perm(n);
    for (uint32_t i = 0; i < n; ++i) { perm[i].key = score_key(s[i]); perm[i].idx = i; }
    std::sort(perm.begin(), perm.end(), [](const Ranked& a, const Ranked& b) {
        if (a.key != b.key) return a.key > b.key;
        return a.idx < b.idx;
    });
    uint32_t tkey = perm[k - 1].key;
    uint32_t n_gt = 0;
    for (uint32_t i = 0; i < n; ++i) if (perm[i].key > tkey) ++n_gt;
    if (thr) { thr->key = tkey; thr->n_gt = n_gt; thr->n_eq_take = k - n_gt; }
    std::vector<uint32_t> chosen(k);
    for (uint32_t j = 0; j < k; ++j) chosen[j] = perm[j].idx;
    std::sort(chosen.begin(), chosen.end());
    for (uint32_t j = 0; j < k; ++j) idx_out[j] = chosen[j];
    return 0;
}

// The value half of O4: the accumulated residual itself, copied bit for bit.
void oracle_take(const float* r, const uint32_t* idx, uint32_t k, float* val) {
    for (uint32_t j = 0; j < k; ++j) std::memcpy(&val[j], &r[idx[j]], sizeof(float));
}

// The rank of element i under (score descending, index ascending), by counting:
// the number of elements that come before it.  Element i is selected iff its
// rank is < k.  O(n) per call, no sort: the route by which single outputs are
// checked at sizes where the full sort is too slow.
uint64_t oracle_rank_of(const float* s, uint64_t n, uint64_t i) {
    uint32_t ki = score_key(s[i]);
    uint64_t before = 0;
    for (uint64_t j = 0; j < n; ++j) {
        uint32_t kj = score_key(s[j]);
        if (kj > ki || (kj == ki && j < i)) ++before;
    }
    return before;
}

// O1..O4 for one layer on one worker.  k == 0: accumulate only.
int oracle_compress_layer(const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                          uint32_t* idx_out, float* val_out, oracle_threshold* thr) {
    if (k > n) return -1;
    oracle_accumulate(r, g, n);
    if (k == 0) return 0;
    std::vector<float> s(n);
    oracle_score(w, r, n, eps, s.data());
    int rc = oracle_select(s.data(), n, k, idx_out, thr);
    if (rc) return rc;
    oracle_take(r, idx_out, k, val_out);
    return 0;
}

// O2..O3 without the accumulate: the threshold record of a layer.
int oracle_select_threshold(const float* w, const float* r, uint32_t n, uint32_t k, float eps,
                            oracle_threshold* thr) {
    if (k > n || k == 0) return -1;
    std::vector<float> s(n);
    std::vector<uint32_t> idx(k);
    oracle_score(w, r, n, eps, s.data());
    return oracle_select(s.data(), n, k, idx.data(), thr);
}

// O5.  Fixed left fold over the workers, starting from worker 0's value.
void oracle_gather_sum(const float* const* residuals, uint32_t W, const uint32_t* idx, uint64_t k,
                       float* sum) {
    for (uint64_t j = 0; j < k; ++j) {
        float acc = residuals[0][idx[j]];
        for (uint32_t p = 1; p < W; ++p) acc = acc + residuals[p][idx[j]];
        sum[j] = acc;
    }
}

// O6 then O7.  Product rounded, then sum rounded; sent residuals become +0.
void oracle_apply_sparse_update(float* w, const uint32_t* idx, const float* sum, uint64_t k, float scale,
                                float* const* residuals, uint32_t W) {
    for (uint64_t j = 0; j < k; ++j) {
        float t = scale * sum[j];
        w[idx[j]] = w[idx[j]] + t;
    }
    for (uint32_t p = 0; p < W; ++p)
        for (uint64_t j = 0; j < k; ++j) residuals[p][idx[j]] = 0.0f;
}

// One whole emulated step over a flat parameter set (Alg. 1, one iteration of
// the outer loop): every worker accumulates every layer; the leader of each
// layer scores, selects and emits its pairs (global flat positions, ascending
// within the layer, layers in table order); then reduce, update and clear over
// the concatenated index list.  pairs_total = sum of k over the table.
// accumulate[p] == 0 skips O1 for worker p (a peer whose residual is static).
int oracle_step(float* w, const float* const* g, float* const* r, const uint8_t* accumulate, float momentum, uint32_t W,
                const oracle_layer* layers, const uint32_t* leader, uint32_t n_layers, float eps,
                float scale, uint32_t* idx_out, float* val_out, float* sum_out, oracle_threshold* thr_out) {
    uint64_t pairs_total = 0;
    for (uint32_t j = 0; j < n_layers; ++j) {
        const oracle_layer& L = layers[j];
        if (L.k > L.n) return -1;
        if (L.out_offset != pairs_total) return -3;  // pairs of the layers are packed back to back
        for (uint32_t p = 0; p < W; ++p) {
            if (accumulate && !accumulate[p]) continue;
            oracle_accumulate_momentum(r[p] + L.offset, g[p] + L.offset, L.n, momentum);
        }
        if (L.k == 0) continue;
        uint32_t lead = leader[j];
        if (lead >= W) return -2;
        std::vector<float> s(L.n);
        oracle_score(w + L.offset, r[lead] + L.offset, L.n, eps, s.data());
        uint32_t* idx = idx_out + L.out_offset;
        int rc = oracle_select(s.data(), L.n, L.k, idx, thr_out ? &thr_out[j] : nullptr);
        if (rc) return rc;
        oracle_take(r[lead] + L.offset, idx, L.k, val_out + L.out_offset);
        for (uint32_t q = 0; q < L.k; ++q) idx[q] += (uint32_t)L.offset;  // local -> flat position
        pairs_total += L.k;
    }
    std::vector<const float*> rc_ptrs(r, r + W);
    oracle_gather_sum(rc_ptrs.data(), W, idx_out, pairs_total, sum_out);
    oracle_apply_sparse_update(w, idx_out, sum_out, pairs_total, scale, r, W);
    return 0;
}


// ------------------------------------------------------------------ threshold mode

// Bytes of one layer's encoded mask: whole 32-bit words.
uint64_t oracle_mask_bytes(uint64_t n) { return ((n + 31) / 32) * 4; }

// T1 + T2 for one chosen node: scores above thr, strictly; bit i%8 of byte i/8.
void oracle_mask_threshold(const float* w, const float* r, uint64_t n, float eps, float thr, uint8_t* mask) {
    std::memset(mask, 0, oracle_mask_bytes(n));
    for (uint64_t i = 0; i < n; ++i) {
        float denom = std::fabs(w[i]) + eps;
        float s = std::fabs(r[i]) / denom;
        if (s > thr) mask[i >> 3] = (uint8_t)(mask[i >> 3] | (1u << (i & 7)));
    }
}

// T3: acc |= m, byte by byte.
void oracle_mask_or(uint8_t* acc, const uint8_t* m, uint64_t nbytes) {
    for (uint64_t b = 0; b < nbytes; ++b) acc[b] = (uint8_t)(acc[b] | m[b]);
}

// The masked positions of a layer in ascending order; returns how many.
uint64_t oracle_mask_indices(const uint8_t* mask, uint64_t n, uint32_t* idx_out) {
    uint64_t c = 0;
    for (uint64_t i = 0; i < n; ++i)
        if ((mask[i >> 3] >> (i & 7)) & 1u) idx_out[c++] = (uint32_t)i;
    return c;
}

// S1: Philox-4x32-10.
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// S1: the uniform draw of element i of a layer at a step.
float oracle_uniform(uint64_t seed, uint64_t step, uint32_t layer, uint32_t i) {
    const uint32_t ctr[4] = {i >> 2, layer, (uint32_t)step, (uint32_t)(step >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return (float)(out[i & 3u] >> 8) * 0x1p-24f;
}

// S2 (with T2's encoding): above the threshold, or drawn with probability s / thr.
void oracle_mask_threshold_random(const float* w, const float* r, uint64_t n, float eps, float thr, uint64_t seed,
                                  uint64_t step, uint32_t layer, uint8_t* mask) {
    std::memset(mask, 0, oracle_mask_bytes(n));
    for (uint64_t i = 0; i < n; ++i) {
        float denom = std::fabs(w[i]) + eps;
        float s = std::fabs(r[i]) / denom;
        float p = s / thr;
        float u = oracle_uniform(seed, step, layer, (uint32_t)i);
        if (s > thr || u < p) mask[i >> 3] = (uint8_t)(mask[i >> 3] | (1u << (i & 7)));
    }
}

}  // extern "C"

namespace {
struct RandomSelection { uint64_t seed, step; };

// One whole iteration of Algorithm 1 in threshold mode on a flat parameter set.
// leaders: n_layers x n_lead chosen nodes per layer (row-major); thr: one threshold
// per layer; mask_out: the layers' encoded masks back to back (oracle_mask_bytes(n)
// each); count_out[j]: masked positions of layer j; idx_out / sum_out: the masked
// flat positions of all layers packed in table order and the reduced values, at most
// max_pairs (returns -4 if there are more).  Every worker with accumulate[p] != 0
// adds its gradient first; every worker is cleared at the masked positions.
int step_threshold_impl(float* w, const float* const* g, float* const* r, const uint8_t* accumulate, float momentum,
                        uint32_t W,
                        const oracle_layer* layers, const uint32_t* leaders, uint32_t n_lead, const float* thr,
                        uint32_t thr_per_slot, const RandomSelection* rs, uint32_t n_layers, float eps, float scale,
                        uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out, float* sum_out, uint64_t max_pairs,
                        uint64_t* total_out) {
    uint64_t total = 0, mask_off = 0;
    for (uint32_t j = 0; j < n_layers; ++j) {
        const oracle_layer& L = layers[j];
        for (uint32_t p = 0; p < W; ++p) {
            if (accumulate && !accumulate[p]) continue;
            oracle_accumulate_momentum(r[p] + L.offset, g[p] + L.offset, L.n, momentum);
        }
        const uint64_t nbytes = oracle_mask_bytes(L.n);
        uint8_t* mask = mask_out + mask_off;
        std::memset(mask, 0, nbytes);
        std::vector<uint8_t> one(nbytes);
        for (uint32_t q = 0; q < n_lead; ++q) {
            const uint32_t lead = leaders[(size_t)j * n_lead + q];
            if (lead >= W) return -2;
            const float t = thr_per_slot ? thr[(size_t)j * n_lead + q] : thr[j];
            if (rs)
                oracle_mask_threshold_random(w + L.offset, r[lead] + L.offset, L.n, eps, t, rs->seed, rs->step, j,
                                             one.data());
            else
                oracle_mask_threshold(w + L.offset, r[lead] + L.offset, L.n, eps, t, one.data());
            oracle_mask_or(mask, one.data(), nbytes);
        }
        std::vector<uint32_t> local(L.n);
        const uint64_t c = oracle_mask_indices(mask, L.n, local.data());
        count_out[j] = (uint32_t)c;
        if (total + c > max_pairs) return -4;
        for (uint64_t q = 0; q < c; ++q) idx_out[total + q] = (uint32_t)(L.offset + local[q]);
        total += c;
        mask_off += nbytes;
    }
    if (total_out) *total_out = total;
    std::vector<const float*> rc_ptrs(r, r + W);
    oracle_gather_sum(rc_ptrs.data(), W, idx_out, total, sum_out);
    oracle_apply_sparse_update(w, idx_out, sum_out, total, scale, r, W);
    return 0;
}
}  // namespace

extern "C" {

// thr_per_slot != 0: thr holds n_layers x n_lead values, one per chosen node.
int oracle_step_threshold(float* w, const float* const* g, float* const* r, const uint8_t* accumulate, float momentum,
                          uint32_t W,
                          const oracle_layer* layers, const uint32_t* leaders, uint32_t n_lead,
                          const float* thr, uint32_t thr_per_slot, uint32_t n_layers, float eps, float scale,
                          uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out, float* sum_out,
                          uint64_t max_pairs, uint64_t* total_out) {
    return step_threshold_impl(w, g, r, accumulate, momentum, W, layers, leaders, n_lead, thr, thr_per_slot, nullptr, n_layers,
                               eps, scale, mask_out, count_out, idx_out, sum_out, max_pairs, total_out);
}

// The same step with random gradient selection (S1, S2) on every chosen node.
int oracle_step_threshold_random(float* w, const float* const* g, float* const* r, const uint8_t* accumulate,
                                 float momentum, uint32_t W, const oracle_layer* layers, const uint32_t* leaders, uint32_t n_lead,
                                 const float* thr, uint32_t thr_per_slot, uint64_t seed, uint64_t step,
                                 uint32_t n_layers, float eps, float scale, uint8_t* mask_out, uint32_t* count_out,
                                 uint32_t* idx_out, float* sum_out, uint64_t max_pairs, uint64_t* total_out) {
    const RandomSelection rs{seed, step};
    return step_threshold_impl(w, g, r, accumulate, momentum, W, layers, leaders, n_lead, thr, thr_per_slot, &rs, n_layers, eps,
                               scale, mask_out, count_out, idx_out, sum_out, max_pairs, total_out);
}

// ------------------------------------------------------------------ layer-wise threshold

// L1: mean and population variance of one node's importance values over a layer.
void oracle_layer_stats(const float* w, const float* r, uint64_t n, float eps, double* mean_out, double* var_out) {
    if (n == 0) { *mean_out = 0.0; *var_out = 0.0; return; }
    std::vector<float> s(n);
    oracle_score(w, r, n, eps, s.data());
    double sum = 0.0;
    for (uint64_t i = 0; i < n; ++i) sum += (double)s[i];
    const double mean = sum / (double)n;
    double m2 = 0.0;
    for (uint64_t i = 0; i < n; ++i) {
        const double d = (double)s[i] - mean;
        m2 += d * d;
    }
    *mean_out = mean;
    *var_out = m2 / (double)n;
}

// L2: the threshold Eq. 4 derives from the statistics.
float oracle_layerwise_threshold(double mean, double var, double alpha, double beta, double C) {
    const double ratio = var / mean;
    const double t = ratio > C ? alpha + beta * ratio : alpha - beta * ratio;
    return (float)t;
}

// One whole iteration with layer-wise thresholds: accumulate, L1 + L2 on every chosen node
// (stats_out: n_layers x n_lead x {mean, var}; thr_out: n_layers x n_lead), then the
// threshold-mode step with those thresholds.
int oracle_step_layerwise(float* w, const float* const* g, float* const* r, const uint8_t* accumulate, float momentum,
                          uint32_t W,
                          const oracle_layer* layers, const uint32_t* leaders, uint32_t n_lead, double alpha,
                          double beta, double C, uint32_t n_layers, float eps, float scale, double* stats_out,
                          float* thr_out, uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out,
                          float* sum_out, uint64_t max_pairs, uint64_t* total_out) {
    for (uint32_t j = 0; j < n_layers; ++j) {
        const oracle_layer& L = layers[j];
        for (uint32_t p = 0; p < W; ++p) {
            if (accumulate && !accumulate[p]) continue;
            oracle_accumulate_momentum(r[p] + L.offset, g[p] + L.offset, L.n, momentum);
        }
        for (uint32_t q = 0; q < n_lead; ++q) {
            const uint32_t lead = leaders[(size_t)j * n_lead + q];
            if (lead >= W) return -2;
            double mean, var;
            oracle_layer_stats(w + L.offset, r[lead] + L.offset, L.n, eps, &mean, &var);
            stats_out[2 * ((size_t)j * n_lead + q)] = mean;
            stats_out[2 * ((size_t)j * n_lead + q) + 1] = var;
            thr_out[(size_t)j * n_lead + q] = oracle_layerwise_threshold(mean, var, alpha, beta, C);
        }
    }
    std::vector<uint8_t> none(W, 0);                 // everything is accumulated already
    return oracle_step_threshold(w, g, r, none.data(), 1.0f, W, layers, leaders, n_lead, thr_out, 1, n_layers, eps, scale,
                                 mask_out, count_out, idx_out, sum_out, max_pairs, total_out);
}

}  // extern "C"
