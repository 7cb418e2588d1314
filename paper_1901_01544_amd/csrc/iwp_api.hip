// Host side of the C ABI declared in include/iwp.h: argument checks, workspace
// carving and the launch sequences.  Every compute step runs in the kernels of
// iwp_select.hpp / iwp_exchange.hpp; nothing here touches element data and
// nothing falls back to the CPU.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "iwp_common.hpp"
#include "iwp_exchange.hpp"
#include "iwp_select.hpp"

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

#define IWP_LAUNCHED(name)                                    \
    do {                                                      \
        hipError_t e_ = hipGetLastError();                    \
        if (e_ != hipSuccess) return hip_fail(e_, name);      \
    } while (0)

// Optional timing of one named kernel with HIP events on the stream it is launched
// on (iwp_timing_*): off by default, costs one string compare per launch when on.
struct Timing {
    static constexpr int MAX = 8192;
    bool enabled = false;
    char name[64] = "";
    std::vector<hipEvent_t> start, stop;
    int used = 0;
    int dropped = 0;
} g_timing;

struct TimedLaunch {       // records an event pair around the launches made while it is alive
    hipStream_t s;
    int slot = -1;
    TimedLaunch(const char* kernel, hipStream_t stream) : s(stream) {
        if (!g_timing.enabled || strcmp(kernel, g_timing.name) != 0) return;
        if (g_timing.used >= (int)g_timing.start.size()) { ++g_timing.dropped; return; }
        slot = g_timing.used++;
        (void)hipEventRecord(g_timing.start[slot], s);
    }
    ~TimedLaunch() {
        if (slot >= 0) (void)hipEventRecord(g_timing.stop[slot], s);
    }
};

inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~size_t(255); }
inline uint32_t tiles_of(uint32_t n) { return (uint32_t)(((uint64_t)n + TILE - 1) / TILE); }

// Carving of a caller-supplied workspace.
struct Workspace {
    DevLayer* single_table;   // 2 rows, used by the single-layer entry points
    uint32_t* hist;           // n_layers * HIST_BINS
    LayerState* state;        // n_layers
    uint2* counts;            // tiles
    size_t bytes;
};

Workspace carve(void* base, uint32_t n_layers, uint32_t tiles) {
    Workspace ws;
    char* p = static_cast<char*>(base);
    size_t off = 0;
    ws.single_table = reinterpret_cast<DevLayer*>(p + off);   off += round256(2 * sizeof(DevLayer));
    ws.hist = reinterpret_cast<uint32_t*>(p + off);           off += round256((size_t)n_layers * HIST_BINS * sizeof(uint32_t));
    ws.state = reinterpret_cast<LayerState*>(p + off);        off += round256((size_t)n_layers * sizeof(LayerState));
    ws.counts = reinterpret_cast<uint2*>(p + off);            off += round256((size_t)tiles * sizeof(uint2));
    ws.bytes = off;
    return ws;
}

struct Table {                // what the kernels need to know about a layer table
    const DevLayer* layers;   // device, n_layers rows + sentinel
    uint32_t n_layers;
    uint32_t tiles;           // per worker
    bool any_k;
};

int check_eps(float eps) { return (eps >= 0.0f && std::isfinite(eps)) ? IWP_OK : IWP_EINVAL; }

// Selection + compaction on the leaders' residuals, after look 1 has filled the
// first-digit histograms (from_thr == nullptr), or from given threshold records.
int run_select_compact(const Table& T, const Workspace& ws, const ResidualPtrs& R, const float* w,
                       const uint32_t* leader, uint32_t W, float eps, const iwp_threshold* from_thr, bool do_compact,
                       uint32_t* idx_out, float* val_out, iwp_threshold* thr_out, hipStream_t s) {
    if (!T.any_k || T.tiles == 0) return IWP_OK;
    if (from_thr == nullptr) {
        {
            TimedLaunch tl_("k_pick<0>", s);
            k_pick<0><<<T.n_layers, BLOCK, 0, s>>>(T.layers, ws.hist, ws.state, thr_out);
        }
        IWP_LAUNCHED("k_pick<0>");
        {
            TimedLaunch tl_("k_refine_hist<1>", s);
            k_refine_hist<1><<<T.tiles, BLOCK, 0, s>>>(R, w, T.layers, T.n_layers, leader, W, eps, ws.state, ws.hist);
        }
        IWP_LAUNCHED("k_refine_hist<1>");
        {
            TimedLaunch tl_("k_pick<1>", s);
            k_pick<1><<<T.n_layers, BLOCK, 0, s>>>(T.layers, ws.hist, ws.state, thr_out);
        }
        IWP_LAUNCHED("k_pick<1>");
        {
            TimedLaunch tl_("k_refine_hist<2>", s);
            k_refine_hist<2><<<T.tiles, BLOCK, 0, s>>>(R, w, T.layers, T.n_layers, leader, W, eps, ws.state, ws.hist);
        }
        IWP_LAUNCHED("k_refine_hist<2>");
        {
            TimedLaunch tl_("k_pick<2>", s);
            k_pick<2><<<T.n_layers, BLOCK, 0, s>>>(T.layers, ws.hist, ws.state, thr_out);
        }
        IWP_LAUNCHED("k_pick<2>");
    } else {
        {
            TimedLaunch tl_("k_load_thresholds", s);
            k_load_thresholds<<<(T.n_layers + BLOCK - 1) / BLOCK, BLOCK, 0, s>>>(T.layers, T.n_layers, from_thr, ws.state);
        }
        IWP_LAUNCHED("k_load_thresholds");
    }
    if (!do_compact) return IWP_OK;
    {
        TimedLaunch tl_("k_tile_count", s);
        k_tile_count<<<T.tiles, BLOCK, 0, s>>>(R, w, T.layers, T.n_layers, leader, W, eps, ws.state, ws.counts);
    }
    IWP_LAUNCHED("k_tile_count");
    {
        TimedLaunch tl_("k_tile_scan", s);
        k_tile_scan<<<T.n_layers, BLOCK, 0, s>>>(T.layers, ws.counts);
    }
    IWP_LAUNCHED("k_tile_scan");
    {
        TimedLaunch tl_("k_compact_write", s);
        k_compact_write<<<T.tiles, BLOCK, 0, s>>>(R, w, T.layers, T.n_layers, leader, W, eps, ws.state, ws.counts, idx_out, val_out);
    }
    IWP_LAUNCHED("k_compact_write");
    return IWP_OK;
}

int launch_init(const Workspace& ws, uint32_t n_layers, bool single, uint32_t n, uint32_t k, hipStream_t s) {
    const uint64_t words = (uint64_t)n_layers * HIST_BINS;
    uint32_t grid = (uint32_t)std::min<uint64_t>((words + BLOCK - 1) / BLOCK, 4096);
    if (grid == 0) grid = 1;
    {
        TimedLaunch tl_("k_init", s);
        k_init<<<grid, BLOCK, 0, s>>>(ws.hist, words, single ? ws.single_table : nullptr, n, k);
    }
    IWP_LAUNCHED("k_init");
    return IWP_OK;
}

}  // namespace

struct iwp_plan {
    std::vector<iwp_layer> rows;
    DevLayer* dev = nullptr;      // n_layers + 1 rows
    uint32_t n_layers = 0;
    uint32_t tiles = 0;
    uint64_t pairs = 0;
    bool any_k = false;
    size_t ws_bytes = 0;
};

extern "C" {

const char* iwp_strerror(int code) {
    switch (code) {
        case IWP_OK: return "ok";
        case IWP_EINVAL: return "invalid argument";
        case IWP_EALIGN: return "buffer not 4-byte aligned";
        case IWP_EWORKSPACE: return "workspace missing or too small";
        case IWP_ERANGE: return "layer does not fit the 32-bit index range";
        case IWP_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* iwp_last_hip_error(void) { return g_hip_error; }

size_t iwp_workspace_bytes(uint32_t n) { return carve(nullptr, 1, tiles_of(n)).bytes; }

// ----------------------------------------------------------------- single layer

static int single_common(const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                         const iwp_threshold* from_thr, bool do_compact, uint32_t* idx_out, float* val_out,
                         iwp_threshold* thr_out, void* workspace, size_t workspace_bytes, hipStream_t s) {
    if (k > n) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (n > IWP_MAX_FLAT) return IWP_ERANGE;
    if (n == 0) return IWP_OK;
    if (!r || (k > 0 && !w) || (k > 0 && do_compact && (!idx_out || !val_out))) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(g) || !aligned4(r) || !aligned4(idx_out) || !aligned4(val_out) ||
        !aligned4(thr_out) || !aligned4(from_thr))
        return IWP_EALIGN;
    const uint32_t tiles = tiles_of(n);
    Workspace ws = carve(workspace, 1, tiles);
    if (!workspace || workspace_bytes < ws.bytes) return IWP_EWORKSPACE;   // holds the one-row layer table too
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return IWP_EALIGN;

    WorkerPtrs P;
    memset(&P, 0, sizeof P);
    P.g[0] = g;
    P.r[0] = r;
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = r;
    int rc = launch_init(ws, 1, true, n, k, s);
    if (rc) return rc;
    Table T{ws.single_table, 1, tiles, k > 0};
    if (from_thr == nullptr) {
        {
            TimedLaunch tl_("k_accumulate_hist", s);
            k_accumulate_hist<<<tiles, BLOCK, 0, s>>>(P, w, T.layers, 1, tiles, nullptr, 1, eps, ws.hist);
        }
        IWP_LAUNCHED("k_accumulate_hist");
    }
    return run_select_compact(T, ws, R, w, nullptr, 1, eps, from_thr, do_compact, idx_out, val_out, thr_out, s);
}

int compress_layer(const float* w, const float* g, float* r, uint32_t n, uint32_t k, float eps,
                   uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n > 0 && !g) return IWP_EINVAL;
    return single_common(w, g, r, n, k, eps, nullptr, true, idx_out, val_out, nullptr, workspace, workspace_bytes,
                         static_cast<hipStream_t>(hip_stream));
}

int select_threshold(const float* w, const float* r, uint32_t n, uint32_t k, float eps, iwp_threshold* thr_out,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (k == 0 || !thr_out) return IWP_EINVAL;
    // r is only read: no gradient pointer means no accumulation
    return single_common(w, nullptr, const_cast<float*>(r), n, k, eps, nullptr, false, nullptr, nullptr, thr_out,
                         workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

int compact_pairs(const float* w, const float* r, uint32_t n, float eps, const iwp_threshold* thr, uint32_t k,
                  uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (k == 0 || !thr) return IWP_EINVAL;
    return single_common(w, nullptr, const_cast<float*>(r), n, k, eps, thr, true, idx_out, val_out, nullptr,
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
    {
        TimedLaunch tl_("k_gather_sum", static_cast<hipStream_t>(hip_stream));
        k_gather_sum<<<(k + BLOCK - 1) / BLOCK, BLOCK, 0, static_cast<hipStream_t>(hip_stream)>>>(R, W, idx, k, sum_out);
    }
    IWP_LAUNCHED("k_gather_sum");
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
    {
        TimedLaunch tl_("k_apply_update", static_cast<hipStream_t>(hip_stream));
        k_apply_update<<<(k + BLOCK - 1) / BLOCK, BLOCK, 0, static_cast<hipStream_t>(hip_stream)>>>(w, idx, sum, k, scale, R, W);
    }
    IWP_LAUNCHED("k_apply_update");
    return IWP_OK;
}

// ----------------------------------------------------------------- plans and segmented calls

int iwp_plan_create(const iwp_layer* layers, uint32_t n_layers, iwp_plan** plan_out) {
    if (!plan_out) return IWP_EINVAL;
    *plan_out = nullptr;
    if (!layers || n_layers == 0) return IWP_EINVAL;
    std::vector<DevLayer> dev(n_layers + 1);
    uint64_t pairs = 0, tiles = 0, end = 0;
    bool any_k = false;
    for (uint32_t j = 0; j < n_layers; ++j) {
        const iwp_layer& L = layers[j];
        if (L.offset < 0 || L.k > L.n) return IWP_EINVAL;
        if ((uint64_t)L.offset < end) return IWP_EINVAL;              // table order, no overlap
        if ((uint64_t)L.offset + L.n > IWP_MAX_FLAT) return IWP_ERANGE;
        if (L.out_offset != pairs) return IWP_EINVAL;                  // packed outputs
        dev[j].offset = (uint64_t)L.offset;
        dev[j].n = L.n;
        dev[j].k = L.k;
        dev[j].out_offset = L.out_offset;
        dev[j].tile_begin = (uint32_t)tiles;
        end = (uint64_t)L.offset + L.n;
        pairs += L.k;
        tiles += tiles_of(L.n);
        any_k = any_k || L.k > 0;
        if (pairs > 0xFFFFFFFFull || tiles > 0x7FFFFFFFull / IWP_MAX_WORKERS) return IWP_ERANGE;
    }
    dev[n_layers] = DevLayer{0, 0, 0, (uint32_t)pairs, (uint32_t)tiles};
    iwp_plan* plan = new (std::nothrow) iwp_plan;
    if (!plan) return IWP_EINVAL;
    plan->rows.assign(layers, layers + n_layers);
    plan->n_layers = n_layers;
    plan->tiles = (uint32_t)tiles;
    plan->pairs = pairs;
    plan->any_k = any_k;
    plan->ws_bytes = carve(nullptr, n_layers, (uint32_t)tiles).bytes;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&plan->dev), dev.size() * sizeof(DevLayer));
    if (e == hipSuccess) e = hipMemcpy(plan->dev, dev.data(), dev.size() * sizeof(DevLayer), hipMemcpyHostToDevice);
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

size_t iwp_plan_workspace_bytes(const iwp_plan* plan) { return plan ? plan->ws_bytes : 0; }
uint64_t iwp_plan_total_pairs(const iwp_plan* plan) { return plan ? plan->pairs : 0; }

static int check_ws(const iwp_plan* plan, void* workspace, size_t workspace_bytes) {
    if (!workspace || workspace_bytes < plan->ws_bytes) return IWP_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return IWP_EALIGN;
    return IWP_OK;
}

int compress_segmented(const iwp_plan* plan, const float* w, const float* const* g, float* const* r, uint32_t W,
                       const uint32_t* leader, float eps, uint32_t* idx_out, float* val_out, iwp_threshold* thr_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!plan || !g || !r || W == 0 || W > IWP_MAX_WORKERS) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (plan->any_k && (!w || !idx_out || !val_out)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(idx_out) || !aligned4(val_out) || !aligned4(thr_out) || !aligned4(leader))
        return IWP_EALIGN;
    WorkerPtrs P;
    memset(&P, 0, sizeof P);
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    for (uint32_t p = 0; p < W; ++p) {
        if (!r[p]) return IWP_EINVAL;
        if (!aligned4(r[p]) || !aligned4(g[p])) return IWP_EALIGN;
        P.g[p] = g[p];
        P.r[p] = r[p];
        R.r[p] = r[p];
    }
    int rc = check_ws(plan, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->tiles == 0) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Workspace ws = carve(workspace, plan->n_layers, plan->tiles);
    rc = launch_init(ws, plan->n_layers, false, 0, 0, s);
    if (rc) return rc;
    Table T{plan->dev, plan->n_layers, plan->tiles, plan->any_k};
    {
        TimedLaunch tl_("k_accumulate_hist", s);
        k_accumulate_hist<<<W * plan->tiles, BLOCK, 0, s>>>(P, w, T.layers, T.n_layers, T.tiles, leader, W, eps, ws.hist);
    }
    IWP_LAUNCHED("k_accumulate_hist");
    return run_select_compact(T, ws, R, w, leader, W, eps, nullptr, true, idx_out, val_out, thr_out, s);
}

int select_threshold_segmented(const iwp_plan* plan, const float* w, const float* r, float eps,
                               iwp_threshold* thr_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!plan || !w || !r || !thr_out) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(thr_out)) return IWP_EALIGN;
    int rc = check_ws(plan, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->tiles == 0 || !plan->any_k) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Workspace ws = carve(workspace, plan->n_layers, plan->tiles);
    rc = launch_init(ws, plan->n_layers, false, 0, 0, s);
    if (rc) return rc;
    WorkerPtrs P;
    memset(&P, 0, sizeof P);
    P.r[0] = const_cast<float*>(r);       // no gradient pointer: the residual is only read
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = const_cast<float*>(r);
    Table T{plan->dev, plan->n_layers, plan->tiles, plan->any_k};
    {
        TimedLaunch tl_("k_accumulate_hist", s);
        k_accumulate_hist<<<plan->tiles, BLOCK, 0, s>>>(P, w, T.layers, T.n_layers, T.tiles, nullptr, 1, eps, ws.hist);
    }
    IWP_LAUNCHED("k_accumulate_hist");
    return run_select_compact(T, ws, R, w, nullptr, 1, eps, nullptr, false, nullptr, nullptr, thr_out, s);
}

int compact_pairs_segmented(const iwp_plan* plan, const float* w, const float* r, float eps, const iwp_threshold* thr,
                            uint32_t* idx_out, float* val_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
    if (!plan || !w || !r || !thr) return IWP_EINVAL;
    if (check_eps(eps)) return IWP_EINVAL;
    if (plan->any_k && (!idx_out || !val_out)) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(thr) || !aligned4(idx_out) || !aligned4(val_out)) return IWP_EALIGN;
    int rc = check_ws(plan, workspace, workspace_bytes);
    if (rc) return rc;
    if (plan->tiles == 0 || !plan->any_k) return IWP_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    Workspace ws = carve(workspace, plan->n_layers, plan->tiles);
    ResidualPtrs R;
    memset(&R, 0, sizeof R);
    R.r[0] = const_cast<float*>(r);
    Table T{plan->dev, plan->n_layers, plan->tiles, plan->any_k};
    return run_select_compact(T, ws, R, w, nullptr, 1, eps, thr, true, idx_out, val_out, nullptr, s);
}

// ----------------------------------------------------------------- helpers

int iwp_copy_f32(float* dst, const float* src, uint64_t n, void* hip_stream) {
    if (n == 0) return IWP_OK;
    if (!dst || !src) return IWP_EINVAL;
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return IWP_EALIGN;
    const uint64_t quads = n / 4;
    uint32_t grid = (uint32_t)std::min<uint64_t>((quads + (uint64_t)BLOCK * 4 - 1) / ((uint64_t)BLOCK * 4), 1u << 20);
    if (grid == 0) grid = 1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    {
        TimedLaunch tl_("k_copy", s);
        k_copy<<<grid, BLOCK, 0, s>>>(dst, src, n);
    }
    IWP_LAUNCHED("k_copy");
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
    g_timing.dropped = 0;
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

int iwp_score_keys(const float* w, const float* r, uint32_t n, float eps, uint32_t* key_out, void* hip_stream) {
    if (check_eps(eps)) return IWP_EINVAL;
    if (n == 0) return IWP_OK;
    if (!w || !r || !key_out) return IWP_EINVAL;
    if (!aligned4(w) || !aligned4(r) || !aligned4(key_out)) return IWP_EALIGN;
    uint32_t grid = (uint32_t)std::min<uint64_t>(((uint64_t)n + BLOCK - 1) / BLOCK, 65536);
    {
        TimedLaunch tl_("k_score_keys", static_cast<hipStream_t>(hip_stream));
        k_score_keys<<<grid, BLOCK, 0, static_cast<hipStream_t>(hip_stream)>>>(w, r, n, eps, key_out);
    }
    IWP_LAUNCHED("k_score_keys");
    return IWP_OK;
}

}  // extern "C"
