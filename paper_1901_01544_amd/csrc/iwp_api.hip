// Host side of the C ABI declared in include/iwp.h: argument checks, workspace
// carving and the launch sequences.  Every compute step runs in the kernels of
// iwp_stream.hpp / iwp_select.hpp / iwp_exchange.hpp; nothing here touches element
// data and nothing falls back to the CPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "iwp_common.hpp"
#include "iwp_exchange.hpp"
#include "iwp_select.hpp"
#include "iwp_stream.hpp"
#include "iwp_threshold.hpp"

using namespace iwp;

namespace {

thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e, const char* what) {
    snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", what, hipGetErrorString(e));
    return IWP_EHIP;
}

#define IWP_HIP(call)                                         \
    do {                                                      \
        hipError_t e_ = (call);                               \
        if (e_ != hipSuccess) return hip_fail(e_, #call);     \
    } while (0)

// Optional timing of one named kernel with HIP events on the stream it is launched
// on (iwp_timing_*): off by default, costs one string compare per launch when on.
struct Timing {
    static constexpr int MAX = 8192;
    bool enabled = false;
    char name[64] = "";
    std::vector<hipEvent_t> start, stop;
    int used = 0;
} g_timing;

struct TimedLaunch {       // records an event pair around the launch made while it is alive
    hipStream_t s;
    int slot = -1;
    TimedLaunch(const char* kernel, hipStream_t stream) : s(stream) {
        if (!g_timing.enabled || strcmp(kernel, g_timing.name) != 0) return;
        if (g_timing.used >= (int)g_timing.start.size()) return;
        slot = g_timing.used++;
        (void)hipEventRecord(g_timing.start[slot], s);
    }
    ~TimedLaunch() {
        if (slot >= 0) (void)hipEventRecord(g_timing.stop[slot], s);
    }
};

// Launch `kernel<<<grid, BLOCK, 0, s>>>(args...)`, timed if asked for, and turn a
// launch failure into IWP_EHIP.
#define IWP_LAUNCH(name, kernel, grid, s, ...)                        \
    do {                                                              \
        {                                                             \
            TimedLaunch tl_(name, s);                                 \
            kernel<<<(grid), BLOCK, 0, (s)>>>(__VA_ARGS__);           \
        }                                                             \
        hipError_t e_ = hipGetLastError();                            \
        if (e_ != hipSuccess) return hip_fail(e_, name);              \
    } while (0)

// Scratch of compress_segmented_static: device memory that belongs to the library, one copy per
// GPU, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and fills are given the address that call returns, looked up once
// per device with that device current.
static __device__ __align__(256) unsigned char scratch[IWP_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch(void** out) {
    int dev = -1;
    IWP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return IWP_EINVAL;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        IWP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return IWP_EALIGN;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return IWP_OK;
}

inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~size_t(255); }
inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + TILE - 1) / TILE); }
inline uint32_t stiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + STILE - 1) / STILE); }
// Staging entries per tile of a layer: three times the number of kept elements an
// average tile holds, plus room for the threshold bin.  A tile that overflows its
// slot is re-read by the later passes instead, which is exact as well.
inline uint32_t slot_cap_of(uint32_t n, uint32_t k) {
    if (k == 0) return 0u;
    const uint64_t per_tile = ((uint64_t)TILE * k + n - 1) / n;
    return (uint32_t)std::min<uint64_t>(TILE, 64 + 3 * per_tile);
}

// Copies of a layer's first-digit histogram: one per FLUSHES_PER_COPY look-1 workgroups, a power of two.
inline uint32_t h0_copies_of(uint32_t n, uint32_t k) {
    if (k == 0) return 1u;
    const uint32_t groups = (tiles_of(n) + LGROUP - 1) / LGROUP;
    uint32_t c = 1;
    while (c < MAX_H0_COPIES && c * FLUSHES_PER_COPY < groups) c <<= 1;
    return c;
}

struct Sizes {                // everything the workspace layout depends on
    uint32_t n_layers, tiles, stiles;
    uint64_t pairs, slots;    // slots: staging entries over all tiles
    uint64_t mask_words;      // 32-bit words of all layers' encoded masks (threshold mode)
    uint64_t hist_words;      // words of all layers' histograms
    uint32_t W_gather;        // rows of the gather matrix (whole-step entry point), else 0
};

// Carving of a caller-supplied workspace.
struct Workspace {
    DevLayer* single_table;   // 2 rows, used by the single-layer entry points
    uint64_t hist_words;      // what k_init clears
    uint32_t* hist;           // hist_words
    LayerState* state;        // n_layers
    uint32_t* stage;          // tiles: staged entries per tile, or RAW_TILE
    uint2* tile_counts;       // tiles
    uint2* stile_counts;      // stiles
    uint32_t* tile_out;       // tiles
    StageArrays A;            // `slots` entries each
    float* gathered;          // W_gather * pairs
    size_t bytes;
};

Workspace carve(void* base, const Sizes& z) {
    Workspace ws;
    const uintptr_t b = reinterpret_cast<uintptr_t>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { uintptr_t p = b + off; off += round256(bytes); return p; };
    ws.single_table = reinterpret_cast<DevLayer*>(take(2 * sizeof(DevLayer)));
    const size_t hist_bytes = round256((size_t)z.hist_words * sizeof(uint32_t));
    const size_t state_bytes = round256((size_t)z.n_layers * sizeof(LayerState));
    ws.hist = reinterpret_cast<uint32_t*>(take(hist_bytes));
    ws.state = reinterpret_cast<LayerState*>(take(state_bytes));
    ws.hist_words = z.hist_words;
    ws.stage = reinterpret_cast<uint32_t*>(take((size_t)z.tiles * sizeof(uint32_t)));
    ws.tile_counts = reinterpret_cast<uint2*>(take((size_t)z.tiles * sizeof(uint2)));
    ws.stile_counts = reinterpret_cast<uint2*>(take((size_t)z.stiles * sizeof(uint2)));
    ws.tile_out = reinterpret_cast<uint32_t*>(take((size_t)z.tiles * sizeof(uint32_t)));
    ws.A.key = reinterpret_cast<uint32_t*>(take(z.slots * sizeof(uint32_t)));
    ws.A.idx = reinterpret_cast<uint32_t*>(take(z.slots * sizeof(uint32_t)));
    ws.A.val = reinterpret_cast<float*>(take(z.slots * sizeof(float)));
    ws.gathered = reinterpret_cast<float*>(take((size_t)z.W_gather * z.pairs * sizeof(float)));
    ws.bytes = off;
    return ws;
}

struct Table {                // what the launches need to know about a layer table
    const DevLayer* layers;   // device, n_layers rows + sentinel
    uint32_t n_layers, tiles, stiles;
    uint64_t pairs;
    bool any_k;
    uint32_t max_layer_stiles;   // super-tiles of the longest layer
};

// Up to this many super-tiles per layer (128 Mi elements) k_write adds up the earlier super-tiles'
// counts itself (16 loads per thread at most); beyond, a scan launch is cheaper.
constexpr uint32_t FOLD_SCAN_MAX_STILES = 4096;

int check_eps(float eps) { return (eps >= 0.0f && std::isfinite(eps)) ? IWP_OK : IWP_EINVAL; }

// Sampling source of a call: the leaders' residuals and gradients (NULL entries allowed), or nothing.
SampleSource sample_from(const WorkerPtrs& P, const float* w, const uint32_t* leader, uint32_t W, float eps) {
    SampleSource S;
    S.P = P; S.w = w; S.leader = leader; S.W = W; S.eps = eps; S.on = w ? 1u : 0u;
    return S;
}

int launch_init(const Workspace& ws, uint32_t n_layers, const iwp_threshold* hint, const DevLayer* layers,
                const DevLayer* row, const DevLayer* sentinel, const SampleSource& S, hipStream_t s) {
    uint32_t zero_blocks = (uint32_t)std::min<uint64_t>((ws.hist_words + BLOCK - 1) / BLOCK, 4096);
    if (zero_blocks == 0) zero_blocks = 1;
    DevLayer zero;
    memset(&zero, 0, sizeof zero);
    IWP_LAUNCH("k_init", k_init, n_layers + zero_blocks, s, ws.hist, ws.hist_words, ws.state, n_layers, hint, layers,
               row ? ws.single_table : nullptr, row ? *row : zero, sentinel ? *sentinel : zero, S);
    return IWP_OK;
}

enum Stop { STOP_AT_THRESHOLD, FULL };

// Selection on the leaders' residuals after look 1 has filled the first-digit
// histograms, then (FULL) the ordered split.  fused: whole-step route (leader row
// of the gather matrix, leader residual cleared).
// Workgroups of look 1: one per tile, or GROUP / LGROUP per super-tile when a workgroup takes several tiles.
constexpr uint32_t leader_grid(uint32_t tiles, uint32_t stiles) {
    return LGROUP == 1 ? tiles : stiles * (GROUP / LGROUP);
}

// Up to these table sizes (bytes of one flat buffer's share of the table) look 1 leaves the weights, or the weights
// and the residual it writes, in the memory-side cache for the kernels that come back to them (see lead_tile).
constexpr uint64_t KEEP_W_AND_R_MAX_BYTES = 104ull << 20, KEEP_W_MAX_BYTES = 160ull << 20;

int launch_leader_pass(const Table& T, const Workspace& ws, const WorkerPtrs& P, const float* w, const uint32_t* leader,
                       uint32_t W, float eps, hipStream_t s) {
    const uint32_t grid = leader_grid(T.tiles, T.stiles);
    const uint64_t bytes = (uint64_t)T.tiles * TILE * sizeof(float);
    if (bytes <= KEEP_W_AND_R_MAX_BYTES) {
        IWP_LAUNCH("k_leader_pass", (k_leader_pass<LGROUP, KEEP_W_AND_R>), grid, s, P, w, T.layers, T.n_layers, leader, W,
                   eps, ws.hist, ws.state, ws.stage, ws.A);
    } else if (bytes <= KEEP_W_MAX_BYTES) {
        IWP_LAUNCH("k_leader_pass", (k_leader_pass<LGROUP, KEEP_W>), grid, s, P, w, T.layers, T.n_layers, leader, W, eps,
                   ws.hist, ws.state, ws.stage, ws.A);
    } else {
        IWP_LAUNCH("k_leader_pass", (k_leader_pass<LGROUP, KEEP_NOTHING>), grid, s, P, w, T.layers, T.n_layers, leader, W,
                   eps, ws.hist, ws.state, ws.stage, ws.A);
    }
    return IWP_OK;
}

template <bool FUSED>
int launch_write(const Table& T, const Workspace& ws, const ResidualPtrs& R, const float* w, const uint32_t* leader,
                 uint32_t W, float eps, bool all_raw, uint32_t* idx_out, float* val_out, hipStream_t s) {
    const uint32_t grid = T.stiles * (GROUP / (BLOCK / WAVE));
    float* gathered = FUSED ? ws.gathered : nullptr;
    if (T.max_layer_stiles <= FOLD_SCAN_MAX_STILES) {
        IWP_LAUNCH("k_write", (k_write<FUSED, true>), grid, s, R, w, T.layers, T.n_layers, leader, W, eps, ws.state,
                   ws.stage, ws.A, all_raw, ws.tile_counts, ws.stile_counts, ws.tile_out, idx_out, val_out, gathered,
                   T.pairs);
    } else {
        IWP_LAUNCH("k_scan", k_scan, T.n_layers, s, T.layers, ws.stile_counts, false, nullptr);
        IWP_LAUNCH("k_write", (k_write<FUSED, false>), grid, s, R, w, T.layers, T.n_layers, leader, W, eps, ws.state,
                   ws.stage, ws.A, all_raw, ws.tile_counts, ws.stile_counts, ws.tile_out, idx_out, val_out, gathered,
                   T.pairs);
    }
    return IWP_OK;
}

// Selection on the leaders' residuals after look 1 has filled the first-digit
// histograms, then (FULL) the ordered split.  fused: whole-step route (leader row
// of the gather matrix, leader residual cleared).
int run_select(const Table& T, const Workspace& ws, const ResidualPtrs& R, const float* w, const uint32_t* leader,
               uint32_t W, float eps, Stop stop, bool fused, uint32_t* idx_out, float* val_out,
               iwp_threshold* thr_out, hipStream_t s) {
    if (!T.any_k || T.tiles == 0) return IWP_OK;
    IWP_LAUNCH("k_first_pick", k_first_pick, T.n_layers, s, T.layers, ws.hist, ws.state);
    // Consecutive tiles per workgroup: STAGE_TILES on tables of long layers (most tiles have nothing to do when look 1
    // staged their layer), one on tables of short layers (a layer that has to be read again wants all the workgroups
    // it can get), more on tables of very long layers (fewer flushes into a layer's one histogram), at most 64 (their
    // look-1 counts are fetched one per lane).
    const uint32_t avg_tiles = T.tiles / std::max<uint32_t>(1u, T.n_layers);
    const uint32_t per_wg = avg_tiles < STAGE_LONG_LAYER_TILES ? 1u :
        std::min<uint32_t>(std::max<uint32_t>(avg_tiles / STAGE_TILES_PER_AVG, STAGE_TILES), STAGE_TILES_MAX);
    const uint32_t stage_grid = std::max<uint32_t>(std::min<uint32_t>((T.tiles + per_wg - 1) / per_wg, STAGE_MAX_GRID),
                                                   (T.tiles + WAVE - 1) / WAVE);
    IWP_LAUNCH("k_stage", k_stage, stage_grid, s, R, w, T.layers, T.n_layers, T.tiles,
               leader, W, eps, ws.state, ws.hist, ws.stage, ws.A);
    const uint32_t stile_grid = std::min<uint32_t>(T.stiles, STILE_MAX_GRID);
    IWP_LAUNCH("k_refine2", k_refine2, stile_grid, s, R, w, T.layers, T.n_layers, T.stiles, leader, W, eps, ws.state,
               ws.stage, ws.A, ws.hist);
    if (stop == STOP_AT_THRESHOLD) {
        IWP_LAUNCH("k_final_pick", k_final_pick, T.n_layers, s, T.layers, ws.hist, ws.state, thr_out);
        return IWP_OK;
    }
    IWP_LAUNCH("k_count", k_count<false>, stile_grid, s, R, w, T.layers, T.n_layers, T.stiles, leader, W, eps, ws.state,
               ws.hist, thr_out, ws.stage, ws.A, ws.tile_counts, ws.stile_counts);
    if (fused) return launch_write<true>(T, ws, R, w, leader, W, eps, false, idx_out, val_out, s);
    return launch_write<false>(T, ws, R, w, leader, W, eps, false, idx_out, val_out, s);
}

// Ordered split from threshold records given by the caller (nothing is staged: every tile is re-read).
int run_compact_from(const Table& T, const Workspace& ws, const ResidualPtrs& R, const float* w, float eps,
                     const iwp_threshold* thr, uint32_t* idx_out, float* val_out, hipStream_t s) {
    if (!T.any_k || T.tiles == 0) return IWP_OK;
    IWP_LAUNCH("k_load_thresholds", k_load_thresholds, (T.n_layers + BLOCK - 1) / BLOCK, s, T.layers, T.n_layers, thr,
               ws.state);
    IWP_LAUNCH("k_count", k_count<true>, std::min<uint32_t>(T.stiles, STILE_MAX_GRID), s, R, w, T.layers, T.n_layers,
               T.stiles, nullptr, 1u, eps, ws.state, ws.hist, nullptr, ws.stage, ws.A, ws.tile_counts, ws.stile_counts);
    return launch_write<false>(T, ws, R, w, nullptr, 1u, eps, true, idx_out, val_out, s);
}

}  // namespace

struct iwp_plan {
    std::vector<iwp_layer> rows;
    DevLayer* dev = nullptr;      // n_layers + 1 rows
    Sizes z{};
    uint64_t flat_end = 0;        // one past the last element any layer covers
    bool any_k = false;
    bool all_k = true;            // every non-empty layer selects something
    uint32_t max_layer_stiles = 0;
    float momentum = 1.0f;        // r <- momentum * r + g in every call that accumulates through this plan
};

extern "C" {

const char* iwp_strerror(int code) {
    switch (code) {
        case IWP_OK: return "ok";
        case IWP_EINVAL: return "invalid argument";
        case IWP_EALIGN: return "buffer not aligned as required";
        case IWP_EWORKSPACE: return "workspace missing or too small";
        case IWP_ERANGE: return "layer does not fit the 32-bit index range";
        case IWP_EHIP: return "HIP runtime error";
        case IWP_ESCRATCH: return "plan needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

const char* iwp_last_hip_error(void) { return g_hip_error; }

// ----------------------------------------------------------------- single layer

static Sizes single_sizes(uint32_t n, uint32_t k) {
    Sizes z;
    z.n_layers = 1; z.tiles = tiles_of(n); z.stiles = stiles_of(n);
    z.pairs = k; z.slots = (uint64_t)z.tiles * slot_cap_of(n, k); z.mask_words = ((uint64_t)n + 31) / 32;
    z.hist_words = layer_hist_words(h0_copies_of(n, k));
    z.W_gather = 0;
    return z;
}

size_t iwp_workspace_bytes(uint32_t n, uint32_t k) { return carve(nullptr, single_sizes(n, std::min(n, k))).bytes; }

enum SingleOp { OP_COMPRESS, OP_SELECT, OP_COMPACT };

static int single_common(SingleOp op, const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                         const iwp_threshold* from_thr, uint32_t* idx_out, float* val_out, iwp_threshold* thr_out,
                         void* workspace, size_t workspace_bytes, hipStream_t s) {
    if (k > n) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (n > IWP_MAX_FLAT) return IWP_ERANGE;
    if (n == 0) return IWP_OK;
    const bool emits = op != OP_SELECT && k > 0;
    if (!r || (k > 0 && !w) || (emits && (!idx_out || !val_out))) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(g) || !aligned4(r) || !aligned4(idx_out) || !aligned4(val_out) ||
        !aligned4(thr_out) || !aligned4(from_thr))
        return IWP_EALIGN;
    const Sizes z = single_sizes(n, k);
    Workspace ws = carve(workspace, z);
    if (!workspace || workspace_bytes < ws.bytes) return IWP_EWORKSPACE;   // holds the one-row layer table too
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return IWP_EALIGN;

    WorkerPtrs P;
    memset(&P, 0, sizeof P);
    P.g[0] = g;
    P.r[0] = r;
    P.momentum = 1.0f;
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = r;
    DevLayer row, sentinel;
    memset(&row, 0, sizeof row);
    memset(&sentinel, 0, sizeof sentinel);
    row.n = n; row.k = k; row.slot_cap = slot_cap_of(n, k);
    row.hist_begin = 0; row.h0_copies = h0_copies_of(n, k);
    sentinel.tile_begin = z.tiles; sentinel.stile_begin = z.stiles; sentinel.out_offset = k;
    SampleSource S = sample_from(P, w, nullptr, 1u, eps);
    if (op == OP_COMPACT || k == 0) S.on = 0;
    int rc = launch_init(ws, 1, nullptr, nullptr, &row, &sentinel, S, s);
    if (rc) return rc;
    Table T{ws.single_table, 1, z.tiles, z.stiles, k, k > 0, z.stiles};
    if (op == OP_COMPACT) return run_compact_from(T, ws, R, w, eps, from_thr, idx_out, val_out, s);
    if (k > 0) {
        rc = launch_leader_pass(T, ws, P, w, nullptr, 1u, eps, s);
        if (rc) return rc;
    } else if (g)
        IWP_LAUNCH("k_accumulate_rest", k_accumulate_rest, z.tiles, s, P, T.layers, 1u, z.tiles, nullptr, 1u);
    return run_select(T, ws, R, w, nullptr, 1u, eps, op == OP_SELECT ? STOP_AT_THRESHOLD : FULL, false, idx_out,
                      val_out, thr_out, s);
}

int compress_layer(const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                   uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n > 0 && !g) return IWP_EINVAL;
    return single_common(OP_COMPRESS, w, g, r, n, k, eps, nullptr, idx_out, val_out, nullptr, workspace,
                         workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int select_threshold(const float* w, const float* r, uint32_t n, uint32_t k, float eps, iwp_threshold* thr_out,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (k == 0 || !thr_out) return IWP_EINVAL;
    // r is only read: no gradient pointer means no accumulation
    return single_common(OP_SELECT, w, nullptr, const_cast<float*>(r), n, k, eps, nullptr, nullptr, nullptr, thr_out,
                         workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int compact_pairs(const float* w, const float* r, uint32_t n, float eps, const iwp_threshold* thr, uint32_t k,
                  uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (k == 0 || !thr) return IWP_EINVAL;
    return single_common(OP_COMPACT, w, nullptr, const_cast<float*>(r), n, k, eps, thr, idx_out, val_out, nullptr,
                         workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

// ----------------------------------------------------------------- exchange

int gather_sum_at_indices(const float* const* residuals, uint32_t W, const uint32_t* idx, uint32_t k,
                          float* sum_out, void* hip_stream) {
    if (W == 0 || W > IWP_MAX_WORKERS || !residuals) return IWP_EINVAL;
    if (k == 0) return IWP_OK;
    if (!idx || !sum_out) return IWP_EINVAL;
    if (!aligned4(idx) || !aligned4(sum_out)) return IWP_EALIGN;
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    for (uint32_t p = 0; p < W; ++p) {
        if (!residuals[p]) return IWP_EINVAL;
        if (!aligned4(residuals[p])) return IWP_EALIGN;
        R.r[p] = const_cast<float*>(residuals[p]);
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    IWP_LAUNCH("k_gather_sum", k_gather_sum, (k + BLOCK - 1) / BLOCK, s, R, W, idx, k, sum_out);
    return IWP_OK;
}

int apply_sparse_update(float* w, const uint32_t* idx, const float* sum, uint32_t k, float scale,
                        float* const* residuals_to_clear, uint32_t W, void* hip_stream) {
    if (W > IWP_MAX_WORKERS || (W > 0 && !residuals_to_clear)) return IWP_EINVAL;
    if (k == 0) return IWP_OK;
    if (!w || !idx || !sum) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(idx) || !aligned4(sum)) return IWP_EALIGN;
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    for (uint32_t p = 0; p < W; ++p) {
        if (!residuals_to_clear[p]) return IWP_EINVAL;
        if (!aligned4(residuals_to_clear[p])) return IWP_EALIGN;
        R.r[p] = residuals_to_clear[p];
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    IWP_LAUNCH("k_apply_update", k_apply_update, (k + BLOCK - 1) / BLOCK, s, w, idx, sum, k, scale, R, W);
    return IWP_OK;
}

// ----------------------------------------------------------------- plans and segmented calls

int iwp_plan_create(const iwp_layer* layers, uint32_t n_layers, iwp_plan** plan_out) {
    if (!plan_out) return IWP_EINVAL;
    *plan_out = nullptr;
    if (!layers || n_layers == 0) return IWP_EINVAL;
    std::vector<DevLayer> dev(n_layers + 1);
    uint64_t pairs = 0, slots = 0, tiles = 0, stiles = 0, end = 0, mask_words = 0, hist_words = 0;
    bool any_k = false, all_k = true;
    uint32_t max_stiles = 0;
    for (uint32_t j = 0; j < n_layers; ++j) {
        const iwp_layer& L = layers[j];
        if (L.offset < 0 || L.k > L.n) return IWP_EINVAL;
        if ((uint64_t)L.offset < end) return IWP_EINVAL;              // table order, no overlap
        if ((uint64_t)L.offset + L.n > IWP_MAX_FLAT) return IWP_ERANGE;
        if (L.out_offset != pairs) return IWP_EINVAL;                  // packed outputs
        DevLayer& D = dev[j];
        memset(&D, 0, sizeof D);
        D.offset = (uint64_t)L.offset;
        D.slot_begin = slots;
        D.n = L.n;
        D.k = L.k;
        D.out_offset = L.out_offset;
        D.tile_begin = (uint32_t)tiles;
        D.stile_begin = (uint32_t)stiles;
        D.slot_cap = slot_cap_of(L.n, L.k);
        D.mask_begin = (uint32_t)mask_words;
        D.hist_begin = (uint32_t)hist_words;
        D.h0_copies = h0_copies_of(L.n, L.k);
        hist_words += layer_hist_words(D.h0_copies);
        end = (uint64_t)L.offset + L.n;
        pairs += L.k;
        slots += (uint64_t)tiles_of(L.n) * D.slot_cap;
        tiles += tiles_of(L.n);
        stiles += stiles_of(L.n);
        mask_words += ((uint64_t)L.n + 31) / 32;
        any_k = any_k || L.k > 0;
        max_stiles = std::max(max_stiles, stiles_of(L.n));
        if (L.n > 0 && L.k == 0) all_k = false;
        if (pairs > 0xFFFFFFFFull || tiles > 0x7FFFFFFFull / IWP_MAX_WORKERS || hist_words > 0xFFFFFFFFull) return IWP_ERANGE;
    }
    DevLayer& S = dev[n_layers];
    memset(&S, 0, sizeof S);
    S.out_offset = (uint32_t)pairs;
    S.tile_begin = (uint32_t)tiles;
    S.stile_begin = (uint32_t)stiles;
    S.slot_begin = slots;
    iwp_plan* plan = new (std::nothrow) iwp_plan;
    if (!plan) return IWP_EINVAL;
    plan->rows.assign(layers, layers + n_layers);
    plan->z = Sizes{n_layers, (uint32_t)tiles, (uint32_t)stiles, pairs, slots, mask_words, hist_words, 0};
    plan->any_k = any_k;
    plan->all_k = all_k;
    plan->max_layer_stiles = max_stiles;
    plan->flat_end = end;
    // the table, then the layer of every tile and of every super-tile (find_layer reads them)
    std::vector<uint32_t> map;
    map.reserve(tiles + stiles);
    for (uint32_t j = 0; j < n_layers; ++j) map.insert(map.end(), tiles_of(layers[j].n), j);
    for (uint32_t j = 0; j < n_layers; ++j) map.insert(map.end(), stiles_of(layers[j].n), j);
    const size_t table_bytes = dev.size() * sizeof(DevLayer), map_bytes = map.size() * sizeof(uint32_t);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&plan->dev), table_bytes + std::max<size_t>(map_bytes, 4));
    if (e == hipSuccess) e = hipMemcpy(plan->dev, dev.data(), table_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess && map_bytes)
        e = hipMemcpy(reinterpret_cast<char*>(plan->dev) + table_bytes, map.data(), map_bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (plan->dev) (void)hipFree(plan->dev);
        delete plan;
        return hip_fail(e, "iwp_plan_create");
    }
    *plan_out = plan;
    return IWP_OK;
}

void iwp_plan_destroy(iwp_plan* plan) {
    if (!plan) return;
    if (plan->dev) (void)hipFree(plan->dev);
    delete plan;
}

int iwp_plan_set_momentum(iwp_plan* plan, float momentum) {
    if (!plan || !std::isfinite(momentum)) return IWP_EINVAL;
    plan->momentum = momentum;
    return IWP_OK;
}

size_t iwp_plan_workspace_bytes(const iwp_plan* plan) { return plan ? carve(nullptr, plan->z).bytes : 0; }

size_t iwp_plan_step_workspace_bytes(const iwp_plan* plan, uint32_t W) {
    if (!plan) return 0;
    Sizes z = plan->z;
    z.W_gather = W;
    return carve(nullptr, z).bytes;
}

uint64_t iwp_plan_total_pairs(const iwp_plan* plan) { return plan ? plan->z.pairs : 0; }

static int check_ws(size_t need, void* workspace, size_t workspace_bytes) {
    if (!workspace || workspace_bytes < need) return IWP_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return IWP_EALIGN;
    return IWP_OK;
}

static int worker_tables(const float* const* g, float* const* r, uint32_t W, float momentum, WorkerPtrs* P,
                         ResidualPtrs* R) {
    if (!g || !r || W == 0 || W > IWP_MAX_WORKERS) return IWP_EINVAL;
    memset(P, 0, sizeof *P);
    memset(R, 0, sizeof *R);
    P->momentum = momentum;
    for (uint32_t p = 0; p < W; ++p) {
        if (!r[p]) return IWP_EINVAL;
        if (!aligned4(r[p]) || !aligned4(g[p])) return IWP_EALIGN;
        P->g[p] = g[p];
        P->r[p] = r[p];
        R->r[p] = r[p];
    }
    return IWP_OK;
}

// compress_segmented on a workspace that is either the caller's or the library's static scratch.
static int compress_segmented_on(const iwp_plan* plan, const float* w, const float* const* g, float* const* r,
                                 uint32_t W, const uint32_t* leader, const iwp_threshold* thr_hint, float eps,
                                 uint32_t* idx_out, float* val_out, iwp_threshold* thr_out, bool own_scratch,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!plan) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (plan->any_k && (!w || !idx_out || !val_out)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(idx_out) || !aligned4(val_out) || !aligned4(thr_out) || !aligned4(leader) ||
        !aligned4(thr_hint))
        return IWP_EALIGN;
    if (thr_hint && thr_hint == thr_out) return IWP_EINVAL;   // the hint is read while the records are written
    WorkerPtrs P;
    ResidualPtrs R;
    int rc = worker_tables(g, r, W, plan->momentum, &P, &R);
    if (rc) return rc;
    if (own_scratch) {
        // the size check comes first: a plan that does not fit is turned away before anything is looked up
        if (carve(nullptr, plan->z).bytes > IWP_STATIC_SCRATCH_BYTES) return IWP_ESCRATCH;
        rc = static_scratch(&workspace);
        if (rc) return rc;
        workspace_bytes = IWP_STATIC_SCRATCH_BYTES;
    }
    Workspace ws = carve(workspace, plan->z);
    rc = check_ws(ws.bytes, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->z.tiles == 0) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    rc = launch_init(ws, plan->z.n_layers, thr_hint, plan->dev, nullptr, nullptr, sample_from(P, w, leader, W, eps), s);
    if (rc) return rc;
    Table T{plan->dev, plan->z.n_layers, plan->z.tiles, plan->z.stiles, plan->z.pairs, plan->any_k, plan->max_layer_stiles};
    if (T.any_k) {
        rc = launch_leader_pass(T, ws, P, w, leader, W, eps, s);
        if (rc) return rc;
    }
    if (W > 1 || !plan->all_k)
        IWP_LAUNCH("k_accumulate_rest", k_accumulate_rest, W * T.tiles, s, P, T.layers, T.n_layers, T.tiles, leader, W);
    return run_select(T, ws, R, w, leader, W, eps, FULL, false, idx_out, val_out, thr_out, s);
}

int compress_segmented(const iwp_plan* plan, const float* w, const float* const* g, float* const* r, uint32_t W,
                       const uint32_t* leader, const iwp_threshold* thr_hint, float eps, uint32_t* idx_out,
                       float* val_out, iwp_threshold* thr_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
    return compress_segmented_on(plan, w, g, r, W, leader, thr_hint, eps, idx_out, val_out, thr_out, false, workspace,
                                 workspace_bytes, hip_stream);
}

int compress_segmented_static(const iwp_plan* plan, const float* w, const float* const* g, float* const* r,
                              uint32_t W, const uint32_t* leader, const iwp_threshold* thr_hint, float eps,
                              uint32_t* idx_out, float* val_out, iwp_threshold* thr_out, void* hip_stream) {
    return compress_segmented_on(plan, w, g, r, W, leader, thr_hint, eps, idx_out, val_out, thr_out, true, nullptr, 0,
                                 hip_stream);
}

int iwp_step_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                       const uint32_t* leader, const iwp_threshold* thr_hint, float eps, float scale,
                       uint32_t* idx_out, float* val_out, float* sum_out, iwp_threshold* thr_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
    if (!plan) return IWP_EINVAL;
    if (check_eps(eps) || !std::isfinite(scale)) return IWP_EINVAL;
    if (!w) return IWP_EINVAL;
    if (plan->any_k && (!idx_out || !val_out || !sum_out)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(idx_out) || !aligned4(val_out) || !aligned4(sum_out) || !aligned4(thr_out) ||
        !aligned4(leader) || !aligned4(thr_hint))
        return IWP_EALIGN;
    if (thr_hint && thr_hint == thr_out) return IWP_EINVAL;   // the hint is read while the records are written
    WorkerPtrs P;
    ResidualPtrs R;
    int rc = worker_tables(g, r, W, plan->momentum, &P, &R);
    if (rc) return rc;
    Sizes z = plan->z;
    z.W_gather = W;
    Workspace ws = carve(workspace, z);
    rc = check_ws(ws.bytes, workspace, workspace_bytes);
    if (rc) return rc;
    if (z.tiles == 0) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    rc = launch_init(ws, z.n_layers, thr_hint, plan->dev, nullptr, nullptr, sample_from(P, w, leader, W, eps), s);
    if (rc) return rc;
    Table T{plan->dev, z.n_layers, z.tiles, z.stiles, z.pairs, plan->any_k, plan->max_layer_stiles};
    if (T.any_k) {
        rc = launch_leader_pass(T, ws, P, w, leader, W, eps, s);
        if (rc) return rc;
        rc = run_select(T, ws, R, w, leader, W, eps, FULL, true, idx_out, val_out, thr_out, s);
        if (rc) return rc;
    }
    WorkerList acc, stat;                       // workers with / without a gradient
    memset(&acc, 0, sizeof acc);
    memset(&stat, 0, sizeof stat);
    for (uint32_t p = 0; p < W; ++p) {
        if (g[p]) acc.id[acc.n++] = (uint8_t)p; else stat.id[stat.n++] = (uint8_t)p;
    }
    // a single accumulating worker that leads every layer (no leader table: worker 0) has been through look 1 on
    // every tile: nothing follows
    const bool leader_did_all = acc.n == 1 && acc.id[0] == 0 && !leader && plan->all_k;
    if (acc.n && !leader_did_all)
        IWP_LAUNCH("k_follow_gather", k_follow_gather, acc.n * T.tiles, s, P, acc, T.layers, T.n_layers, T.tiles, leader,
                   W, idx_out, ws.tile_out, ws.gathered, T.pairs);
    if (T.any_k) {
        uint32_t static_mask = 0;
        for (uint32_t q = 0; q < stat.n; ++q) static_mask |= 1u << stat.id[q];
        IWP_LAUNCH("k_reduce_update", k_reduce_update, (uint32_t)((T.pairs + BLOCK - 1) / BLOCK), s, R, static_mask, T.layers,
                   T.n_layers, leader, ws.gathered, W, T.pairs, idx_out, w, scale, sum_out, plan->flat_end);
    }
    return IWP_OK;
}

int select_threshold_segmented(const iwp_plan* plan, const float* w, const float* r, float eps,
                               iwp_threshold* thr_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!plan || !w || !r || !thr_out) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(thr_out)) return IWP_EALIGN;
    Workspace ws = carve(workspace, plan->z);
    int rc = check_ws(ws.bytes, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->z.tiles == 0 || !plan->any_k) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    WorkerPtrs P;
    memset(&P, 0, sizeof P);
    P.r[0] = const_cast<float*>(r);       // no gradient pointer: the residual is only read
    P.momentum = 1.0f;
    rc = launch_init(ws, plan->z.n_layers, nullptr, plan->dev, nullptr, nullptr, sample_from(P, w, nullptr, 1u, eps), s);
    if (rc) return rc;
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = const_cast<float*>(r);
    Table T{plan->dev, plan->z.n_layers, plan->z.tiles, plan->z.stiles, plan->z.pairs, plan->any_k, plan->max_layer_stiles};
    rc = launch_leader_pass(T, ws, P, w, nullptr, 1u, eps, s);
    if (rc) return rc;
    return run_select(T, ws, R, w, nullptr, 1u, eps, STOP_AT_THRESHOLD, false, nullptr, nullptr, thr_out, s);
}

int compact_pairs_segmented(const iwp_plan* plan, const float* w, const float* r, float eps, const iwp_threshold* thr,
                            uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    if (!plan || !w || !r || !thr) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (plan->any_k && (!idx_out || !val_out)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(thr) || !aligned4(idx_out) || !aligned4(val_out)) return IWP_EALIGN;
    Workspace ws = carve(workspace, plan->z);
    int rc = check_ws(ws.bytes, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->z.tiles == 0 || !plan->any_k) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = const_cast<float*>(r);
    Table T{plan->dev, plan->z.n_layers, plan->z.tiles, plan->z.stiles, plan->z.pairs, plan->any_k, plan->max_layer_stiles};
    return run_compact_from(T, ws, R, w, eps, thr, idx_out, val_out, s);
}

// ----------------------------------------------------------------- threshold mode

namespace {

struct ThresholdWorkspace {
    uint32_t* lmask;          // n_lead * mask_words
    uint2* tile_counts;       // tiles
    uint2* stile_counts;      // stiles
    uint32_t* tile_out;       // tiles
    uint32_t* layer_total;    // n_layers
    uint32_t* lay_out;        // n_layers + 1
    double2* tile_stats;      // n_lead * tiles (layer-wise thresholds)
    float* gathered;          // W * max_pairs
    size_t bytes;
};

static ThresholdWorkspace carve_threshold(void* base, const Sizes& z, uint32_t W, uint32_t n_lead, uint32_t max_pairs) {
    ThresholdWorkspace ws;
    const uintptr_t b = reinterpret_cast<uintptr_t>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { uintptr_t p = b + off; off += round256(bytes); return p; };
    ws.lmask = reinterpret_cast<uint32_t*>(take((size_t)n_lead * z.mask_words * sizeof(uint32_t)));
    ws.tile_counts = reinterpret_cast<uint2*>(take((size_t)z.tiles * sizeof(uint2)));
    ws.stile_counts = reinterpret_cast<uint2*>(take((size_t)z.stiles * sizeof(uint2)));
    ws.tile_out = reinterpret_cast<uint32_t*>(take((size_t)z.tiles * sizeof(uint32_t)));
    ws.layer_total = reinterpret_cast<uint32_t*>(take((size_t)z.n_layers * sizeof(uint32_t)));
    ws.lay_out = reinterpret_cast<uint32_t*>(take(((size_t)z.n_layers + 1) * sizeof(uint32_t)));
    ws.tile_stats = reinterpret_cast<double2*>(take((size_t)n_lead * z.tiles * sizeof(double2)));
    ws.gathered = reinterpret_cast<float*>(take((size_t)W * max_pairs * sizeof(float)));
    ws.bytes = off;
    return ws;
}

// Rule of the layer-wise threshold; absent (NULL) for caller-supplied thresholds.
struct LayerwiseRule {
    double alpha, beta, C;
    double* stats_out;
    float* thr_out;
};

static int run_threshold_step(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                       const uint32_t* leaders, uint32_t n_lead, const float* thr, const LayerwiseRule* rule,
                       RandomSel rs, float eps, float scale, uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out, float* sum_out,
                       uint32_t max_pairs, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!plan || !w || !leaders || !mask_out || !count_out || !idx_out || !sum_out) return IWP_EINVAL;
    if (n_lead == 0 || n_lead > MAX_LEAD || n_lead > W || max_pairs == 0) return IWP_EINVAL;
    if (check_eps(eps) || !std::isfinite(scale)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(leaders) || !aligned4(thr) || !aligned4(mask_out) || !aligned4(count_out) ||
        !aligned4(idx_out) || !aligned4(sum_out))
        return IWP_EALIGN;
    WorkerPtrs P;
    ResidualPtrs R;
    int rc = worker_tables(g, r, W, plan->momentum, &P, &R);
    if (rc) return rc;
    const Sizes& z = plan->z;
    ThresholdWorkspace ws = carve_threshold(workspace, z, W, n_lead, max_pairs);
    rc = check_ws(ws.bytes, workspace, workspace_bytes);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    uint32_t* mask32 = reinterpret_cast<uint32_t*>(mask_out);
    const DevLayer* layers = plan->dev;
    if (rule) {
        // the chosen nodes accumulate while their statistics are taken; the mask pass then only re-reads
        if (z.tiles)
            IWP_LAUNCH("k_leader_stats", k_leader_stats, n_lead * z.tiles, s, P, w, layers, z.n_layers, z.tiles, leaders,
                       n_lead, W, eps, ws.tile_stats);
        IWP_LAUNCH("k_layer_thr", k_layer_thr, z.n_layers * n_lead, s, layers, z.tiles, leaders, n_lead, W, ws.tile_stats,
                   rule->alpha, rule->beta, rule->C, reinterpret_cast<double2*>(rule->stats_out), rule->thr_out);
        thr = rule->thr_out;
    }
    if (z.tiles) {
        IWP_LAUNCH("k_leader_mask", k_leader_mask, n_lead * z.tiles, s, P, w, layers, z.n_layers, z.tiles, leaders, n_lead, W,
                   thr, rule != nullptr, rule == nullptr, rs, eps, ws.lmask, z.mask_words);
        IWP_LAUNCH("k_mask_or_count", k_mask_or_count, z.stiles, s, layers, z.n_layers, leaders, n_lead, W, ws.lmask,
                   z.mask_words, mask32, ws.tile_counts, ws.stile_counts);
    }
    IWP_LAUNCH("k_scan", k_scan, z.n_layers, s, layers, ws.stile_counts, true, ws.layer_total);
    IWP_LAUNCH("k_layer_offsets", k_layer_offsets, 1u, s, ws.layer_total, z.n_layers, max_pairs, ws.lay_out, count_out);
    if (z.tiles == 0) return IWP_OK;
    IWP_LAUNCH("k_mask_emit", k_mask_emit, (z.tiles + 3) / 4, s, layers, z.n_layers, z.tiles, mask32, ws.tile_counts,
               ws.stile_counts, ws.lay_out, count_out, max_pairs, ws.tile_out, idx_out);
    IWP_LAUNCH("k_follow_mask", k_follow_mask, W * z.tiles, s, P, layers, z.n_layers, z.tiles, leaders, n_lead, W, mask32,
               ws.tile_out, ws.lay_out, count_out, max_pairs, ws.gathered);
    const uint32_t pair_blocks = std::min<uint32_t>((max_pairs + BLOCK - 1) / BLOCK, 8192u);
    IWP_LAUNCH("k_reduce_update_counted", k_reduce_update_counted, pair_blocks, s, P, layers, z.n_layers, leaders, n_lead, W,
               ws.lay_out, count_out, max_pairs, ws.gathered, idx_out, w, scale, sum_out, plan->flat_end);
    return IWP_OK;
}

}  // namespace

size_t iwp_plan_mask_bytes(const iwp_plan* plan) { return plan ? (size_t)plan->z.mask_words * 4 : 0; }

size_t iwp_plan_threshold_workspace_bytes(const iwp_plan* plan, uint32_t W, uint32_t n_lead, uint32_t max_pairs) {
    return plan ? carve_threshold(nullptr, plan->z, W, n_lead, max_pairs).bytes : 0;
}

int iwp_step_threshold_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                                 const uint32_t* leaders, uint32_t n_lead, const float* thr, float eps, float scale,
                                 uint8_t* mask_out, uint32_t* count_out, uint32_t* idx_out, float* sum_out,
                                 uint32_t max_pairs, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!thr) return IWP_EINVAL;
    return run_threshold_step(plan, w, g, r, W, leaders, n_lead, thr, nullptr, RandomSel{0, 0, 0, 0, 0}, eps, scale, mask_out,
                              count_out, idx_out, sum_out, max_pairs, workspace, workspace_bytes, hip_stream);
}

int iwp_step_threshold_random_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r,
                                        uint32_t W, const uint32_t* leaders, uint32_t n_lead, const float* thr,
                                        uint64_t seed, uint64_t step, float eps, float scale, uint8_t* mask_out,
                                        uint32_t* count_out, uint32_t* idx_out, float* sum_out, uint32_t max_pairs,
                                        void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!thr) return IWP_EINVAL;
    const RandomSel rs{1u, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, (uint32_t)(step >> 32)};
    return run_threshold_step(plan, w, g, r, W, leaders, n_lead, thr, nullptr, rs, eps, scale, mask_out, count_out, idx_out,
                              sum_out, max_pairs, workspace, workspace_bytes, hip_stream);
}

int iwp_step_layerwise_segmented(const iwp_plan* plan, float* w, const float* const* g, float* const* r, uint32_t W,
                                 const uint32_t* leaders, uint32_t n_lead, double alpha, double beta, double C, float eps,
                                 float scale, double* stats_out, float* thr_out, uint8_t* mask_out, uint32_t* count_out,
                                 uint32_t* idx_out, float* sum_out, uint32_t max_pairs, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    if (!stats_out || !thr_out) return IWP_EINVAL;
    if (!std::isfinite(alpha) || !std::isfinite(beta) || !std::isfinite(C)) return IWP_EINVAL;
    if ((reinterpret_cast<uintptr_t>(stats_out) & 15u) || !aligned4(thr_out)) return IWP_EALIGN;
    LayerwiseRule rule{alpha, beta, C, stats_out, thr_out};
    return run_threshold_step(plan, w, g, r, W, leaders, n_lead, thr_out, &rule, RandomSel{0, 0, 0, 0, 0}, eps, scale, mask_out, count_out, idx_out,
                              sum_out, max_pairs, workspace, workspace_bytes, hip_stream);
}

// ----------------------------------------------------------------- helpers

int iwp_score_keys(const float* w, const float* r, uint32_t n, float eps, uint32_t* key_out, void* hip_stream) {
    if (check_eps(eps)) return IWP_EINVAL;
    if (n == 0) return IWP_OK;
    if (!w || !r || !key_out) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(key_out)) return IWP_EALIGN;
    uint32_t grid = (uint32_t)std::min<uint64_t>(((uint64_t)n + BLOCK - 1) / BLOCK, 65536);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    IWP_LAUNCH("k_score_keys", k_score_keys, grid, s, w, r, n, eps, key_out);
    return IWP_OK;
}

int iwp_copy_f32(float* dst, const float* src, uint64_t n, void* hip_stream) {
    if (n == 0) return IWP_OK;
    if (!dst || !src) return IWP_EINVAL;
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return IWP_EALIGN;
    const uint64_t blocks = (n / 4 + BLOCK - 1) / BLOCK;
    if (blocks > 0x7FFFFFFFull) return IWP_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    IWP_LAUNCH("k_copy", k_copy, (uint32_t)std::max<uint64_t>(blocks, 1), s, dst, src, n);
    return IWP_OK;
}

int iwp_timing_enable(const char* kernel_name, uint32_t max_launches) {
    if (!kernel_name || strlen(kernel_name) >= sizeof g_timing.name) return IWP_EINVAL;
    if (max_launches == 0 || max_launches > (uint32_t)Timing::MAX) max_launches = Timing::MAX;
    while (g_timing.start.size() < max_launches) {
        hipEvent_t a, b;
        IWP_HIP(hipEventCreate(&a));
        IWP_HIP(hipEventCreate(&b));
        g_timing.start.push_back(a);
        g_timing.stop.push_back(b);
    }
    strcpy(g_timing.name, kernel_name);
    g_timing.used = 0;
    g_timing.enabled = true;
    return IWP_OK;
}

int iwp_timing_collect(double* total_ms, uint32_t* launches) {
    if (!total_ms || !launches) return IWP_EINVAL;
    g_timing.enabled = false;
    double sum = 0.0;
    for (int i = 0; i < g_timing.used; ++i) {
        IWP_HIP(hipEventSynchronize(g_timing.stop[i]));
        float ms = 0.f;
        IWP_HIP(hipEventElapsedTime(&ms, g_timing.start[i], g_timing.stop[i]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (uint32_t)g_timing.used;
    g_timing.used = 0;
    return IWP_OK;
}

}  // extern "C"
