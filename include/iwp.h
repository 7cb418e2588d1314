/*
 * iwp.h -- C ABI of the MI355X (gfx950) library for the per-worker gradient
 * compression step of importance weighted pruning on a ring (arXiv 1901.01544).
 *
 * What the calls compute follows the paper's Algorithm 1 ("Importance Weighted
 * Pruning"): the body of its per-layer loop and the reduce / SGD lines after it,
 * with the importance measure of Section 3.2 (|accumulated gradient / weight|).
 * "Choose threshold" is taken as the exact k-th largest importance of the layer,
 * k being given by the caller as an integer, so every output has a static size.
 * The iwp_step_threshold_* / iwp_step_layerwise_* entry points instead follow the
 * front end as printed -- a fixed threshold per layer (Section 4.1) or one derived
 * from the layer's importance statistics (Section 3.4), masks of several chosen
 * nodes encoded and OR-ed, optional random selection (Section 3.3) -- and report
 * how many elements were sent in device memory.
 *
 * Conventions for every entry point
 *  - All buffer pointers are DEVICE pointers unless the comment says "host".
 *    Pointer tables (g, r, residuals) are host arrays of device pointers.
 *  - fp32 data is IEEE-754 binary32; the library computes in binary32 with
 *    round-to-nearest-even, denormals preserved, correctly rounded divide, no
 *    fused multiply-add.  Indices are uint32.  Inputs must be finite.
 *  - The caller owns every buffer, the workspace included.  The hot-path calls
 *    allocate nothing, free nothing, read nothing back to the host and keep no
 *    state between calls; they only enqueue kernels on `hip_stream` (a
 *    hipStream_t passed as void*, NULL = the default stream) and return, so a
 *    caller may capture them into a HIP graph (scratch is cleared by fill
 *    kernels, never by memset nodes).
 *    Outputs are valid once the stream has been synchronised.  A workspace may be
 *    reused by the next call on the same stream; its contents are scratch.
 *  - Buffers must be 4-byte aligned.  16-byte alignment of (pointer + layer
 *    offset) enables 128-bit accesses; anything else is handled by a slower,
 *    equally exact path.
 *  - Return value: IWP_OK (0) or a negative iwp_status.  Argument errors are
 *    detected before any kernel is launched and leave all buffers untouched.
 *  - Determinism: identical inputs give identical output bytes, run to run.
 *  - Limits: offset + n <= IWP_MAX_FLAT for every layer; W <= IWP_MAX_WORKERS.
 */
#ifndef IWP_H
#define IWP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IWP_MAX_WORKERS 32
#define IWP_MAX_FLAT 0xFFFF0000ull
#define IWP_STATIC_SCRATCH_BYTES (64u << 20)   /* the library's own scratch, see compress_segmented_static */

typedef enum {
    IWP_OK = 0,
    IWP_EINVAL = -1,     /* null pointer, k > n, W out of range, eps negative or NaN, bad table */
    IWP_EALIGN = -2,     /* a buffer is not 4-byte aligned */
    IWP_EWORKSPACE = -3, /* workspace missing or smaller than iwp_*workspace_bytes() */
    IWP_ERANGE = -4,     /* offset + n exceeds IWP_MAX_FLAT */
    IWP_EHIP = -5,       /* a HIP runtime call or a launch failed; see iwp_last_hip_error() */
    IWP_ESCRATCH = -6    /* compress_segmented_static: the plan needs more than IWP_STATIC_SCRATCH_BYTES */
} iwp_status;

/* The threshold of one layer (stands for "choose threshold: thr" of Algorithm 1).
 * key is the bit pattern of the k-th largest importance (sign bit cleared, so
 * unsigned order == float order); n_gt elements lie strictly above it (n_gt < k);
 * of the elements equal to it the n_eq_take = k - n_gt with the lowest indices
 * are kept.  Lives in device memory. */
typedef struct {
    uint32_t key;
    uint32_t n_gt;
    uint32_t n_eq_take;
} iwp_threshold;

/* One row of a layer table (the layers omega[0..M] of Algorithm 1 laid out in
 * flat buffers).  offset: first element of the layer in w / g / r; n: elements;
 * k: elements to keep (0 = accumulate only, nothing selected); out_offset:
 * first (index, value) pair of the layer in idx_out / val_out -- the rows must
 * be packed, out_offset[j] = k[0] + ... + k[j-1]; pad: ignored.  Layers must
 * not overlap. */
typedef struct {
    int64_t offset;
    uint32_t n;
    uint32_t k;
    uint32_t out_offset;
    uint32_t pad;
} iwp_layer;

/* ------------------------------------------------------------------ one layer */

/* Workspace size in bytes for the single-layer calls on a layer of n elements of
 * which k are kept (the staging areas scale with k).  The workspace must be
 * 256-byte aligned. */
size_t iwp_workspace_bytes(uint32_t n, uint32_t k);

/* Algorithm 1, per-layer body on one worker: local accumulation r <- r + g
 * (the accumulation line, read as residual accumulation; Eq. 3), importance
 * |r| / (|w| + eps) of every element (mask line), selection of the k most
 * important elements under (importance descending, index ascending), and the
 * split into the sent part: idx_out[0..k) ascending positions in the layer,
 * val_out[j] = r[idx_out[j]] bit for bit.  r keeps every value (the sent ones are
 * cleared later by apply_sparse_update).  k == 0: accumulate only; idx_out /
 * val_out may then be NULL.  w, g read-only; r read-write; capacity of idx_out,
 * val_out >= k; exactly k pairs are written. */
int compress_layer(const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                   uint32_t* idx_out, float* val_out,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* "Choose threshold" of Algorithm 1 as exact selection, without the accumulate:
 * the threshold record of the layer's importances |r| / (|w| + eps) for 1 <= k <= n,
 * written to thr_out (device). */
int select_threshold(const float* w, const float* r, uint32_t n, uint32_t k, float eps,
                     iwp_threshold* thr_out,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Mask and split lines of Algorithm 1 for a given threshold record `thr` (device,
 * as written by select_threshold for the same w, r, eps, k): emits the k pairs
 * (ascending index, residual value) of the elements above the threshold plus the
 * first thr->n_eq_take elements equal to it. */
int compact_pairs(const float* w, const float* r, uint32_t n, float eps, const iwp_threshold* thr,
                  uint32_t k, uint32_t* idx_out, float* val_out,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ exchange */

/* Arithmetic of the ring all-reduce line of Algorithm 1 on one index set: every
 * worker's residual taken at the leader's indices and summed in the fixed order
 * sum_out[j] = ((R_0[idx_j] + R_1[idx_j]) + ...) + R_{W-1}[idx_j], starting from
 * R_0's value.  residuals: host array of W device pointers (flat buffers that idx
 * indexes); idx: k positions, each < the buffers' length (not checked). */
int gather_sum_at_indices(const float* const* residuals, uint32_t W, const uint32_t* idx, uint32_t k,
                          float* sum_out, void* hip_stream);

/* SGD line of Algorithm 1 / Eq. 3 on the reduced sparse vector, then the
 * "not Mask" line: w[idx_j] <- w[idx_j] + (scale * sum[j]) with the product and
 * the sum each rounded once, and R_p[idx_j] <- +0.0f for the W buffers listed in
 * residuals_to_clear (host array of device pointers; W may be 0).  idx must hold
 * distinct positions (what compaction produces). */
int apply_sparse_update(float* w, const uint32_t* idx, const float* sum, uint32_t k, float scale,
                        float* const* residuals_to_clear, uint32_t W, void* hip_stream);

/* ------------------------------------------------------------------ all layers in one pass */

/* A plan holds a layer table (copied) and its device image.  Creating and
 * destroying a plan are set-up calls: they allocate / free a small device table
 * and synchronise; they are not part of the hot path. */
typedef struct iwp_plan iwp_plan;

/* layers: host array of n_layers rows, validated here (packed out_offsets, k <= n,
 * no overlap in table order, range). */
int iwp_plan_create(const iwp_layer* layers, uint32_t n_layers, iwp_plan** plan_out);
void iwp_plan_destroy(iwp_plan* plan);
/* Momentum-weighted residual (Eq. 3: what is sparsified is m * g_{t-1} + g_t, the residual
 * accumulated locally with momentum).  After this call every entry point that accumulates
 * through the plan (compress_segmented, iwp_step_segmented, iwp_step_threshold_segmented,
 * iwp_step_threshold_random_segmented, iwp_step_layerwise_segmented) computes
 * r[i] <- (m * r[i]) + g[i], the product rounded to binary32, then the sum (never fused).
 * m = 1 (the state of a new plan) is the plain accumulation, bit for bit.  m must be
 * finite.  Host-side state of the plan: takes effect for calls issued afterwards;
 * compress_layer has no plan and always uses m = 1. */
int iwp_plan_set_momentum(iwp_plan* plan, float momentum);

/* Workspace bytes the segmented calls need for this plan (256-byte aligned). */
size_t iwp_plan_workspace_bytes(const iwp_plan* plan);
/* Workspace bytes iwp_step_segmented needs for this plan and W residual buffers. */
size_t iwp_plan_step_workspace_bytes(const iwp_plan* plan, uint32_t W);
/* Sum of k over the plan's layers: the number of pairs the segmented calls emit. */
uint64_t iwp_plan_total_pairs(const iwp_plan* plan);

/* The whole per-layer loop of Algorithm 1 for W workers emulated on one GPU, in a
 * number of launches that does not depend on the layer count.  For every layer j
 * of the plan and every worker p with g[p] != NULL: r[p] <- r[p] + g[p] on the
 * layer's range.  For every layer with k > 0 the worker leader[j] (device array
 * of n_layers entries, each < W; NULL = worker 0 leads everything) is the
 * randomly chosen node of Algorithm 1: its accumulated residual is scored,
 * selected and split exactly as in compress_layer.  Emitted indices are GLOBAL
 * positions in the flat buffers (offset + position in layer), ascending within a
 * layer, layers in table order starting at out_offset; val_out alike.
 * thr_out: device array of n_layers records, or NULL.  w: flat weights; g, r:
 * host arrays of W device pointers to flat buffers with w's layout.
 * thr_hint: NULL or expected thresholds (see iwp_step_segmented); a pure shortcut. */
int compress_segmented(const iwp_plan* plan, const float* w, const float* const* g, float* const* r,
                       uint32_t W, const uint32_t* leader, const iwp_threshold* thr_hint, float eps,
                       uint32_t* idx_out, float* val_out, iwp_threshold* thr_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* compress_segmented for callers that cannot allocate or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors, minus the workspace: the kernels work in a scratch buffer of
 * IWP_STATIC_SCRATCH_BYTES (64 MiB) that is part of the library's device image, so every GPU the
 * library runs on holds one copy until the process ends.  The call allocates and frees nothing
 * (its first call on a device looks the buffer's address up, nothing more).  A plan whose
 * iwp_plan_workspace_bytes() exceeds the buffer is refused with IWP_ESCRATCH before anything is
 * launched (the AlexNet-shaped set needs 46.8 MB, the ResNet-50-shaped one 24.7 MB).  All calls
 * on one GPU share that one buffer, which keeps the last call's contents; each call clears what
 * it needs cleared.  Calls that overlap on one GPU (two streams, two threads) race on it: run them
 * one after the other on one stream, or use compress_segmented with separate workspaces. */
int compress_segmented_static(const iwp_plan* plan, const float* w, const float* const* g, float* const* r,
                              uint32_t W, const uint32_t* leader, const iwp_threshold* thr_hint, float eps,
                              uint32_t* idx_out, float* val_out, iwp_threshold* thr_out, void* hip_stream);

/* One whole iteration of Algorithm 1's outer loop for W workers emulated on one GPU:
 * compress_segmented, gather_sum_at_indices over r[0..W) and apply_sparse_update
 * clearing r[0..W), with the same results bit for bit, but scheduled so that the
 * exchange needs no scattered pass over the residuals: the leaders of all layers
 * are accumulated, scored, selected and split first; the other workers are then
 * accumulated in one streaming pass that also copies their residual at the
 * leader's indices into a W x K gather matrix and leaves +0 behind; a last small
 * kernel sums the W rows in worker order (sum_out, K values), updates
 * w[idx] += scale * sum and is done.  A worker with g[p] == NULL is not accumulated
 * but still gathered and cleared.  Outputs as in the three separate calls:
 * idx_out / val_out (K pairs), sum_out (K), thr_out (n_layers records or NULL);
 * w and every r[p] are updated in place.  Workspace: iwp_plan_step_workspace_bytes.
 * thr_hint: NULL, or a device array of n_layers threshold records that are
 * expected to be close to this call's (typically the previous step's thr_out; a
 * different buffer than thr_out).  The hint never changes any output: it lets the
 * first pass over a leader's layer already copy out every element from slightly
 * below the hinted threshold, which makes the second pass over that layer
 * unnecessary whenever the new threshold is not below that mark; otherwise, and
 * for records that are wrong or garbage, the layer just takes the two-pass route.
 * With NULL the library derives the same mark itself from a small sample of each
 * layer (read-only, inside the call's first launch); equally without influence on
 * any output. */
int iwp_step_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                       const uint32_t* leader, const iwp_threshold* thr_hint, float eps, float scale,
                       uint32_t* idx_out, float* val_out, float* sum_out, iwp_threshold* thr_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* select_threshold for every layer of the plan with k > 0 on one flat residual
 * buffer r; thr_out: device array of n_layers records (rows with k == 0 untouched). */
int select_threshold_segmented(const iwp_plan* plan, const float* w, const float* r, float eps,
                               iwp_threshold* thr_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* compact_pairs for every layer of the plan with k > 0, given thr (device array of
 * n_layers records); global indices as in compress_segmented. */
int compact_pairs_segmented(const iwp_plan* plan, const float* w, const float* r, float eps,
                            const iwp_threshold* thr, uint32_t* idx_out, float* val_out,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ threshold mode */

/* Bytes of the encoded masks of all layers of the plan: layer j's mask takes
 * 4 * ceil(n_j / 32) bytes, the layers follow each other in table order. */
size_t iwp_plan_mask_bytes(const iwp_plan* plan);
size_t iwp_plan_threshold_workspace_bytes(const iwp_plan* plan, uint32_t W, uint32_t n_lead, uint32_t max_pairs);

/* One whole iteration of Algorithm 1 with the front end exactly as printed: a fixed
 * threshold per layer (Section 4.1 uses 0.005 ... 0.1) instead of a k-th largest
 * importance.  For every layer j of the plan (the rows' k and out_offset are not
 * used): every worker with g[p] != NULL accumulates; each of the n_lead chosen nodes
 * leaders[j * n_lead + q] (device array; entries >= W read as 0; a node listed twice
 * counts once) marks the elements with |r| / (|w| + eps) strictly above thr[j]
 * (device array of n_layers floats); the masks are encoded one bit per element
 * (encode_uint8 of Algorithm 1: bit i % 8 of byte i / 8) and OR-ed into mask_out;
 * every worker's residual at the masked positions is summed in worker order,
 * w[i] += scale * sum, and the residuals are cleared there.
 * Outputs: mask_out (iwp_plan_mask_bytes, 4-byte aligned); count_out[0..n_layers) =
 * sent elements per layer, count_out[n_layers] = their total, count_out[n_layers + 1]
 * = 1 if the total exceeds max_pairs -- then the workers are accumulated and the
 * mask and counts are valid, but nothing is exchanged, updated or cleared;
 * idx_out / sum_out (capacity max_pairs): ascending flat positions, layers packed
 * in table order, and the reduced values.  n_lead <= 8 and <= W. */
int iwp_step_threshold_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                                 const uint32_t* leaders, uint32_t n_lead, const float* thr, float eps, float scale,
                                 uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out, float* sum_out,
                                 uint32_t max_pairs, void* workspace, size_t workspace_bytes, void* hip_stream);

/* iwp_step_threshold_segmented with random gradient selection (Section 3.3): on every
 * chosen node an element that is not above the threshold is still marked with
 * probability importance / threshold, to bound the staleness of small gradients.
 * The draw of element i (position inside its layer) of layer j is
 * u = (x >> 8) * 2^-24, x = output word i % 4 of Philox-4x32 with 10 rounds (Salmon et
 * al., SC'11) under key (seed low word, seed high word) and counter (i / 4, j, step low
 * word, step high word); the element is marked iff importance > thr or
 * u < importance / thr (binary32 divide).  The draw does not depend on the node, so a
 * caller can reproduce it.  seed, step: any values; use the iteration number as step.
 * Everything else as in iwp_step_threshold_segmented. */
int iwp_step_threshold_random_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r,
                                        uint32_t W, const uint32_t* leaders, uint32_t n_lead, const float* thr,
                                        uint64_t seed, uint64_t step, float eps, float scale, uint8_t* mask_out,
                                        uint32_t* count_out, uint32_t* idx_out, float* sum_out, uint32_t max_pairs,
                                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same iteration with layer-wise thresholds (Section 3.4, Eq. 4): every chosen node
 * derives its own threshold for the layer from the mean and the (population) variance of
 * its importance values after accumulation:  ratio = var / mean;
 * thr = alpha + beta * ratio if ratio > C, else alpha - beta * ratio  (the two branches of
 * Eq. 4 read by the prose that follows it), evaluated in binary64 and rounded once to
 * binary32; then everything as in iwp_step_threshold_segmented, each node comparing
 * against its own threshold.  alpha, beta, C: the epoch's hyper-parameters, finite.
 * Outputs in addition: stats_out[2 * (j * n_lead + q)] = mean, [.. + 1] = variance
 * (device, 16-byte aligned, binary64) and thr_out[j * n_lead + q] (device, binary32) for
 * the node in slot q of layer j (a node listed twice: same values in both slots).
 * A layer whose importance is zero everywhere has ratio 0/0: its threshold is NaN and
 * nothing of it is sent.  The statistics are sums in binary64 taken in a fixed order
 * (deterministic run to run); they agree with a sequential binary64 evaluation to
 * rounding error of the summation, far inside 1e-6 relative.
 * Workspace: iwp_plan_threshold_workspace_bytes. */
int iwp_step_layerwise_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                                 const uint32_t* leaders, uint32_t n_lead, double alpha, double beta, double C, float eps,
                                 float scale, double* stats_out, float* thr_out, uint8_t* mask_out, uint32_t* count_out,
                                 uint32_t* idx_out, float* sum_out, uint32_t max_pairs, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ helpers */

/* The importance keys exactly as the kernels compute them: key_out[i] = bit
 * pattern of |r[i]| / (|w[i]| + eps) with the sign bit cleared.  For tests of
 * the device arithmetic; not on the hot path. */
int iwp_score_keys(const float* w, const float* r, uint32_t n, float eps, uint32_t* key_out,
                   void* hip_stream);

/* dst[0..n) <- src[0..n), a plain streaming copy with 128-bit accesses (both
 * 16-byte aligned): the measured HBM ceiling that throughput is quoted against
 * and the known-size reference for scaling profiler byte counters. */
int iwp_copy_f32(float* dst, const float* src, uint64_t n, void* hip_stream);

/* Measurement aid, not on the hot path: time every launch of one kernel (by its
 * name, e.g. "k_follow_gather") with HIP event pairs recorded on the stream the
 * kernel is launched on.  enable() creates the events (at most max_launches pairs,
 * 0 = the built-in maximum) and starts recording; collect() stops, waits for the
 * recorded events and returns the summed duration in milliseconds and the number
 * of launches seen.  Process-wide and not thread-safe. */
int iwp_timing_enable(const char* kernel_name, uint32_t max_launches);
int iwp_timing_collect(double* total_ms, uint32_t* launches);

/* Text for a status code; never NULL. */
const char* iwp_strerror(int code);
/* Text of the last HIP error the calling thread hit inside the library ("" if none). */
const char* iwp_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IWP_H */
