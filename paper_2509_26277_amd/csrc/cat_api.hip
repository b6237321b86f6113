// Host driver and C ABI of the CAT hot path (see include/cat.h for the contract).
// Validates arguments, carves the caller's workspace, and enqueues the kernels of
// each step on the caller's stream.  Nothing here synchronises or allocates.
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "cat_common.h"
#include "cat_infer.h"
#include "cat_tile.h"

namespace cat {

static thread_local char g_err[512] = "";
static std::atomic<int> g_path{CAT_PATH_AUTO};
static std::atomic<int> g_early_stop{0};  // cat_allow_early_stop

cat_status set_error(cat_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

// ---- kernel timing (cat_profile_enable / cat_profile_read) -------------------------------
static bool g_prof = false;
static std::vector<hipEvent_t> g_prof_ev;  // pairs (begin, end), reused across enables
static size_t g_prof_used = 0;             // events recorded since the last enable

bool profile_on() { return g_prof; }
bool fast_paths_forced() { return g_path.load() == CAT_PATH_TILE; }
static std::atomic<int> g_apply_kernel{0};  // cat_debug_apply_kernel
static std::atomic<int> g_list_cap{1024};
int lloyd_list_capacity() { return g_list_cap.load(); }
static std::atomic<int> g_queue_cap{256};
int rerank_queue_capacity() { return g_queue_cap.load(); }

cat_status profile_mark(bool begin, hipStream_t st) {
    (void)begin;
    if (g_prof_used == g_prof_ev.size()) {
        hipEvent_t e;
        CAT_HIP_TRY(hipEventCreate(&e));
        g_prof_ev.push_back(e);
    }
    CAT_HIP_TRY(hipEventRecord(g_prof_ev[g_prof_used], st));
    g_prof_used++;
    return CAT_OK;
}

// ---- workspace ------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Carver {
    char* base;
    size_t off = 0;
    explicit Carver(void* b) : base((char*)b) {}
    template <typename T>
    T* take(size_t count) {
        T* p = base ? (T*)(base + off) : nullptr;
        off += align256(count * sizeof(T));
        return p;
    }
};

struct FitWs {
    double* acc;              // 4 x K x D   segmented-sum accumulators
    float* cent[2];           // K x D each  centroid ping-pong
    float* pivx;              // K x D       shifts of the statistics
    float* pivy;              // K x D
    int32_t* counts;          // K
    unsigned long long* rep;  // K           smallest row index of each cluster
    int64_t* idx;             // K           seeded initial rows
    double* inertia;          // 1
    TileWs tile;              // scratch of the MFMA tile kernels
    LloydWs lloyd;            // changed-row list and counters of the fused Lloyd loop
    uint32_t* sort;           // N + 2 K + 2  rows ordered by cluster, for the segmented sums
    size_t bytes;
};

static FitWs carve_fit(void* base, int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    Carver c(base);
    FitWs w;
    size_t KD = (size_t)K * (size_t)D;
    w.acc = c.take<double>(4 * KD);
    w.cent[0] = c.take<float>(KD);
    w.cent[1] = c.take<float>(KD);
    w.pivx = c.take<float>(KD);
    w.pivy = c.take<float>(KD);
    w.counts = c.take<int32_t>(K);
    w.rep = c.take<unsigned long long>(K);
    w.idx = c.take<int64_t>(K);
    w.inertia = c.take<double>(1);
    w.sort = c.take<uint32_t>(sort_workspace_words(N, K));
    size_t tb = tile_workspace_bytes(D, K, dt);
    w.tile = tile_carve(base ? (void*)(c.base + c.off) : nullptr, D, K, dt);
    c.off += align256(tb);
    if (tb) {
        w.lloyd = lloyd_carve(base ? (void*)(c.base + c.off) : nullptr, N, D, K);
        w.lloyd.sort_ws = w.sort;
        c.off += align256(w.lloyd.bytes);
    }
    w.bytes = c.off;
    return w;
}

struct ApplyWs {
    float* g_eff;
    float* b_eff;
    TileWs tile;
    void* split;      // more than 128 clusters ranked by two launches: what the first hands to the second (N pairs), and
    int32_t* labels;  //   the labels the map that follows goes by (N); both only with N given and where that applies
    size_t bytes;
};
// N = 0: without the scratch of the split ranking (cat_apply_static: its array has a fixed size)
static ApplyWs carve_apply(void* base, int64_t D, int32_t K, cat_dtype dt, int64_t N = 0) {
    Carver c(base);
    ApplyWs w;
    size_t KD = (size_t)K * (size_t)D;
    w.g_eff = c.take<float>(KD);
    w.b_eff = c.take<float>(KD);
    size_t tb = tile_workspace_bytes(D, K, dt);
    w.tile = tile_carve(base ? (void*)(c.base + c.off) : nullptr, D, K, dt);
    c.off += align256(tb);
    w.split = nullptr;
    w.labels = nullptr;
    const size_t sb = N > 0 ? tile_split_scratch_bytes(N, D, K, dt) : 0;
    if (sb) {
        w.split = c.take<char>(sb);
        w.labels = c.take<int32_t>((size_t)N);
    }
    w.bytes = c.off;
    return w;
}

// Rows whose length is not a whole number of 16-byte groups do not fit the matrix-core kernels.  A fit reads the rows
// once per Lloyd pass, so it pays to copy them once into rows padded with zero channels (distances are unchanged) and
// to run the clustering on the copy: scratch for the copy, the padded centroids and a fit of the padded shape.
struct PadWs {
    void* lq = nullptr;      // N x Dp rows
    float* cent = nullptr;   // K x Dp
    float* init = nullptr;   // K x Dp
    void* fit = nullptr;     // cat_fit scratch of the padded shape
    void* bounds = nullptr;  // scratch of the bound-based loop on the padded shape (only where asked for)
    int64_t Dp = 0;
    size_t bytes = 0;
};
static int64_t padded_dim(int64_t D, cat_dtype dt) {
    const int64_t step = dt == CAT_BF16 ? 8 : 4;
    return (D + step - 1) / step * step;
}
static bool pad_applies(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    const int64_t Dp = padded_dim(D, dt);
    return Dp != D && !tile_supports(TILE_LLOYD, N, D, K, dt) && tile_supports(TILE_LLOYD, N, Dp, K, dt);
}
// (one pass or none: the copy would cost as much as it saves)
static std::atomic<bool> g_padded_fit{true};  // cat_debug_padded_fit
static bool fit_runs_padded(int64_t N, int64_t D, int32_t K, cat_dtype dt, int32_t iters) {
    return g_padded_fit.load() && g_path.load() == CAT_PATH_AUTO && iters >= 2 && pad_applies(N, D, K, dt);
}
static PadWs carve_pad(void* base, int64_t N, int64_t D, int32_t K, cat_dtype dt, int32_t iters, bool with_bounds) {
    PadWs w;
    w.Dp = padded_dim(D, dt);
    Carver c(base);
    w.lq = c.take<char>((size_t)N * (size_t)w.Dp * (dt == CAT_BF16 ? 2 : 4));
    w.cent = c.take<float>((size_t)K * (size_t)w.Dp);
    w.init = c.take<float>((size_t)K * (size_t)w.Dp);
    w.fit = c.take<char>(carve_fit(nullptr, N, w.Dp, K, dt).bytes);
    if (with_bounds) w.bounds = c.take<char>(bounds_workspace_bytes(N, w.Dp, K, iters));
    w.bytes = c.off;
    return w;
}

// ---- argument checks ----------------------------------------------------------------
static bool shape_ok(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    if (dt != CAT_F32 && dt != CAT_BF16) return false;
    if (N < 1 || D < 1 || K < 1 || (int64_t)K > N || K > CAT_MAX_K) return false;
    if (dt == CAT_BF16 && (D & 1)) return false;
    if (D > (int64_t)1 << 24) return false;
    if (N > ((int64_t)1 << 62) / D) return false;
    return true;
}
static cat_status check_shape(const char* fn, int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt))
        return set_error(CAT_ERR_INVALID_ARG,
                         "%s: need 1 <= K <= min(N, %d), D >= 1 (even for bf16), dt in {F32, BF16}; got N=%lld D=%lld "
                         "K=%d dt=%d",
                         fn, CAT_MAX_K, (long long)N, (long long)D, (int)K, (int)dt);
    return CAT_OK;
}
static cat_status check_ptr(const char* fn, const char* name, const void* p, size_t align) {
    if (!p) return set_error(CAT_ERR_INVALID_ARG, "%s: %s is NULL", fn, name);
    if (((uintptr_t)p) % align) return set_error(CAT_ERR_INVALID_ARG, "%s: %s is not %zu-byte aligned", fn, name, align);
    return CAT_OK;
}
static cat_status check_ws(const char* fn, const void* ws, size_t have, size_t need) {
    if (!ws) return set_error(CAT_ERR_WORKSPACE, "%s: workspace is NULL (need %zu bytes)", fn, need);
    if (((uintptr_t)ws) % 256) return set_error(CAT_ERR_WORKSPACE, "%s: workspace is not 256-byte aligned", fn);
    if (have < need) return set_error(CAT_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", fn, have, need);
    return CAT_OK;
}
#define CAT_TRY(expr)                      \
    do {                                   \
        cat_status _s = (expr);            \
        if (_s != CAT_OK) return _s;       \
    } while (0)

// ---- steps ------------------------------------------------------------------------
// One assignment pass on the selected kernel family.  counts / inertia / rep are optional
// device outputs, initialised here.
static cat_status step_assign(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                              int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                              const TileWs& tw, hipStream_t st, void* split_scratch = nullptr) {
    if (counts) CAT_TRY(launch_fill_zero(counts, (size_t)K * sizeof(int32_t), st));
    if (inertia) CAT_TRY(launch_fill_zero(inertia, sizeof(double), st));
    if (rep) CAT_TRY(launch_fill_u64(rep, K, ~0ull, st));
    const int path = g_path.load();
    const bool tile_ok = tile_supports(TILE_ASSIGN, N, D, K, dt);
    if (path == CAT_PATH_TILE && !tile_ok)
        return set_error(CAT_ERR_UNSUPPORTED, "tile path forced but D=%lld K=%d dt=%d does not fit it", (long long)D,
                         (int)K, (int)dt);
    if (tile_ok && path != CAT_PATH_STREAM) {
        if (split_scratch && tile_split_scratch_bytes(N, D, K, dt))  // more than 128 clusters: two launches of 8 tiles
            return tile_assign_split(lq, dt, N, D, K, cent, assign, counts, inertia, rep, tw, split_scratch, st);
        return tile_assign(lq, dt, N, D, K, cent, assign, counts, inertia, rep, nullptr, nullptr, nullptr, tw, st);
    }
    // shapes outside the matrix-core tile kernels: the row-tile inference kernel without its map where it has an instance
    // (rows that are not whole 16-byte groups), counts and first rows from the labels afterwards; else the LDS streaming
    // kernel; the direct-form kernel only when asked for
    if (path == CAT_PATH_AUTO && assign && tw.packA && infer_supported(N, D, K, dt) && g_apply_kernel.load() != 1) {
        CAT_TRY(infer_apply(lq, dt, N, D, K, cent, nullptr, nullptr, nullptr, assign, tw, st, false, inertia));
        if (counts || rep) CAT_TRY(launch_count_rep(assign, N, K, counts, rep, st));
        return CAT_OK;
    }
    if (path != CAT_PATH_STREAM)
        return launch_assign_lds(lq, dt, N, D, K, cent, assign, counts, inertia, rep, nullptr, nullptr, nullptr, st);
    return launch_assign_stream(lq, dt, N, D, K, cent, assign, counts, inertia, rep, nullptr, nullptr, nullptr, st);
}

static cat_status step_update(const void* lq, cat_dtype dt, const int32_t* assign, int64_t N, int64_t D, int32_t K,
                              const int32_t* counts, const float* prev, float* cent, double* acc, uint32_t* sort_ws,
                              hipStream_t st) {
    CAT_TRY(launch_fill_zero(acc, (size_t)K * D * sizeof(double), st));
    if (segsum_sorted_supported(1, N, D, dt))
        CAT_TRY(launch_segsum_sorted(1, lq, nullptr, dt, assign, counts, N, D, K, nullptr, nullptr, acc, sort_ws, st));
    else
        CAT_TRY(launch_segsum(1, lq, nullptr, dt, assign, N, D, K, nullptr, nullptr, acc, st));
    return launch_finalize_centroids(acc, counts, prev, cent, D, K, st);
}

static cat_status step_stats(const void* lq, const void* fp, cat_dtype dt, const int32_t* assign, int64_t N, int64_t D,
                             int32_t K, const int32_t* counts, const unsigned long long* rep, const float* hint,
                             const FitWs& w, float* gamma, float* beta, hipStream_t st) {
    CAT_TRY(launch_gather_pivots(lq, fp, dt, D, K, rep, hint, w.pivx, w.pivy, st));
    CAT_TRY(launch_fill_zero(w.acc, (size_t)4 * K * D * sizeof(double), st));
    if (segsum_sorted_supported(4, N, D, dt))
        CAT_TRY(launch_segsum_sorted(4, lq, fp, dt, assign, counts, N, D, K, w.pivx, w.pivy, w.acc, w.sort, st));
    else
        CAT_TRY(launch_segsum(4, lq, fp, dt, assign, N, D, K, w.pivx, w.pivy, w.acc, st));
    return launch_finalize_affine(w.acc, counts, w.pivx, w.pivy, gamma, beta, D, K, st);
}

// Initialisation, `iters` Lloyd iterations and the final assignment (everything of cat_fit before the
// affine fit).  Leaves the counts and the first row of every cluster in w.counts / w.rep.  With `skipped`
// given the loop may stop early (see tile_lloyd); the outputs are those of the full loop.
static cat_status run_lloyd(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, int32_t iters, uint64_t seed,
                            const float* init_centroids, float* centroids, int32_t* assignments, double* inertia,
                            const FitWs& w, hipStream_t st, int32_t* skipped = nullptr, const BoundsWs* bw = nullptr) {
    const size_t KD = (size_t)K * (size_t)D;
    const int path = g_path.load();
    const bool fused = tile_supports(TILE_LLOYD, N, D, K, dt) && path != CAT_PATH_STREAM;
    if (path == CAT_PATH_TILE && !fused)
        return set_error(CAT_ERR_UNSUPPORTED, "tile path forced but D=%lld K=%d dt=%d does not fit it", (long long)D,
                         (int)K, (int)dt);
    // init: the fused path iterates in place in the caller's `centroids`
    float* c0 = fused ? centroids : w.cent[0];
    if (init_centroids) {
        CAT_TRY(launch_copy_words(init_centroids, c0, (int64_t)KD, st));
    } else {
        CAT_TRY(launch_init_indices(N, K, seed, w.idx, st));
        CAT_TRY(launch_gather_rows(lq, dt, D, K, w.idx, c0, st));
    }
    if (fused) {
        if (!skipped && g_early_stop.load()) skipped = w.lloyd.skipped;
        // one assignment launch per Lloyd iteration; only the rows that change cluster touch the sums
        CAT_TRY(tile_lloyd(lq, dt, N, D, K, iters, centroids, w.acc, assignments, w.counts, inertia, w.rep, skipped, w.tile, w.lloyd, st, bw));
    } else {
        // the streaming kernels keep no record of the rows that move: every pass runs
        if (skipped) CAT_TRY(launch_fill_zero(skipped, sizeof(int32_t), st));
        int cur = 0;
        for (int32_t t = 0; t < iters; t++) {
            CAT_TRY(step_assign(lq, dt, N, D, K, w.cent[cur], assignments, w.counts, inertia ? w.inertia : nullptr,
                                nullptr, w.tile, st));
            if (inertia) CAT_TRY(launch_copy_words(w.inertia, inertia + t, 2, st));
            CAT_TRY(step_update(lq, dt, assignments, N, D, K, w.counts, w.cent[cur], w.cent[cur ^ 1], w.acc, w.sort, st));
            cur ^= 1;
        }
        // final assignment against the final centroids
        CAT_TRY(step_assign(lq, dt, N, D, K, w.cent[cur], assignments, w.counts, inertia ? w.inertia : nullptr, w.rep,
                            w.tile, st));
        if (inertia) CAT_TRY(launch_copy_words(w.inertia, inertia + iters, 2, st));
        CAT_TRY(launch_copy_words(w.cent[cur], centroids, (int64_t)KD, st));
    }
    return CAT_OK;
}

}  // namespace cat

using namespace cat;

extern "C" {

const char* cat_last_error(void) { return g_err; }

cat_status cat_profile_enable(int on) {
    g_prof = on != 0;
    if (g_prof) g_prof_used = 0;
    return CAT_OK;
}

int cat_profile_read(float* ms_out, int cap) {
    const size_t pairs = g_prof_used / 2;
    for (size_t i = 0; i < pairs; i++) {
        if (hipEventSynchronize(g_prof_ev[2 * i + 1]) != hipSuccess) return -1;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof_ev[2 * i], g_prof_ev[2 * i + 1]) != hipSuccess) return -1;
        if (ms_out && (int)i < cap) ms_out[i] = ms;
    }
    return (int)pairs;
}

cat_status cat_stream_probe(const void* src, void* dst, size_t bytes, void* hip_stream) {
    CAT_TRY(check_ptr("cat_stream_probe", "src", src, 16));
    if (dst) CAT_TRY(check_ptr("cat_stream_probe", "dst", dst, 16));
    if (bytes == 0 || bytes % 16) return set_error(CAT_ERR_INVALID_ARG, "cat_stream_probe: bytes = %zu is not a positive multiple of 16", bytes);
    return launch_stream_probe(src, dst, bytes, (hipStream_t)hip_stream);
}

cat_status cat_debug_list_capacity(int entries) {
    if (entries < 0 || entries > 1024)
        return set_error(CAT_ERR_INVALID_ARG, "cat_debug_list_capacity: %d is outside 0 .. 1024", entries);
    g_list_cap.store(entries == 0 ? 1024 : entries);
    return CAT_OK;
}

cat_status cat_debug_rerank_queue(int entries) {
    if (entries < -1 || entries > 256)
        return set_error(CAT_ERR_INVALID_ARG, "cat_debug_rerank_queue: %d is outside -1 .. 256", entries);
    g_queue_cap.store(entries == 0 ? 256 : (entries < 0 ? 0 : entries));
    return CAT_OK;
}

cat_status cat_debug_apply_kernel(int which) {
    if (which < 0 || which > 2) return set_error(CAT_ERR_INVALID_ARG, "cat_debug_apply_kernel: 0, 1 or 2, got %d", which);
    g_apply_kernel.store(which);
    return CAT_OK;
}

cat_status cat_debug_padded_fit(int on) {
    g_padded_fit.store(on != 0);
    return CAT_OK;
}

cat_status cat_allow_early_stop(int on) {
    g_early_stop.store(on != 0);
    return CAT_OK;
}

cat_status cat_select_path(cat_path p) {
    if (p != CAT_PATH_AUTO && p != CAT_PATH_STREAM && p != CAT_PATH_TILE)
        return set_error(CAT_ERR_INVALID_ARG, "cat_select_path: unknown path %d", (int)p);
    g_path.store((int)p);
    return CAT_OK;
}

size_t cat_fit_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt)) return 0;
    size_t b = carve_fit(nullptr, N, D, K, dt).bytes;
    if (pad_applies(N, D, K, dt)) b = align256(b) + carve_pad(nullptr, N, D, K, dt, 0, false).bytes;
    return b;
}

size_t cat_apply_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt)) return 0;
    return carve_apply(nullptr, D, K, dt, N).bytes;
}

cat_status cat_init_indices(int64_t N, int32_t K, uint64_t seed, int64_t* idx_out) {
    if (N < 1 || K < 1 || (int64_t)K > N || K > CAT_MAX_K || !idx_out)
        return set_error(CAT_ERR_INVALID_ARG, "cat_init_indices: need 1 <= K <= min(N, %d) and idx_out != NULL",
                         CAT_MAX_K);
    const uint64_t cap = init_draw_cap(N);
    int32_t have = 0;
    uint64_t t = 0;
    while (have < K && t < cap) {
        int64_t cand = (int64_t)(splitmix64_at(seed, t) % (uint64_t)N);
        t++;
        bool dup = false;
        for (int32_t q = 0; q < have && !dup; q++) dup = idx_out[q] == cand;
        if (!dup) idx_out[have++] = cand;
    }
    for (int64_t c = 0; have < K && c < N; c++) {
        bool dup = false;
        for (int32_t q = 0; q < have && !dup; q++) dup = idx_out[q] == c;
        if (!dup) idx_out[have++] = c;
    }
    return CAT_OK;
}

cat_status cat_assign(const void* lq, int64_t N, int64_t D, int32_t K, cat_dtype dt, const float* centroids,
                      int32_t* assignments, int32_t* counts, double* inertia, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_shape("cat_assign", N, D, K, dt));
    CAT_TRY(check_ptr("cat_assign", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_assign", "centroids", centroids, 16));
    CAT_TRY(check_ptr("cat_assign", "assignments", assignments, 4));
    FitWs w = carve_fit(workspace, N, D, K, dt);
    CAT_TRY(check_ws("cat_assign", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    return step_assign(lq, dt, N, D, K, centroids, assignments, counts, inertia, nullptr, w.tile, st, w.lloyd.carry);
}

cat_status cat_update(const void* lq, const int32_t* assignments, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                      const float* prev_centroids, float* centroids, int32_t* counts, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_shape("cat_update", N, D, K, dt));
    CAT_TRY(check_ptr("cat_update", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_update", "assignments", assignments, 4));
    CAT_TRY(check_ptr("cat_update", "prev_centroids", prev_centroids, 16));
    CAT_TRY(check_ptr("cat_update", "centroids", centroids, 16));
    FitWs w = carve_fit(workspace, N, D, K, dt);
    CAT_TRY(check_ws("cat_update", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    CAT_TRY(launch_fill_zero(w.counts, (size_t)K * sizeof(int32_t), st));
    CAT_TRY(launch_fill_u64(w.rep, K, ~0ull, st));
    CAT_TRY(launch_count_rep(assignments, N, K, w.counts, w.rep, st));
    CAT_TRY(step_update(lq, dt, assignments, N, D, K, w.counts, prev_centroids, centroids, w.acc, w.sort, st));
    if (counts) CAT_TRY(launch_copy_words(w.counts, counts, K, st));
    return CAT_OK;
}

cat_status cat_stats(const void* lq, const void* fp, const int32_t* assignments, int64_t N, int64_t D, int32_t K,
                     cat_dtype dt, const float* centroids, float* gamma, float* beta, int32_t* counts,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_shape("cat_stats", N, D, K, dt));
    CAT_TRY(check_ptr("cat_stats", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_stats", "fp", fp, 16));
    CAT_TRY(check_ptr("cat_stats", "assignments", assignments, 4));
    CAT_TRY(check_ptr("cat_stats", "gamma", gamma, 16));
    CAT_TRY(check_ptr("cat_stats", "beta", beta, 16));
    if (centroids) CAT_TRY(check_ptr("cat_stats", "centroids", centroids, 16));
    FitWs w = carve_fit(workspace, N, D, K, dt);
    CAT_TRY(check_ws("cat_stats", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    CAT_TRY(launch_fill_zero(w.counts, (size_t)K * sizeof(int32_t), st));
    CAT_TRY(launch_fill_u64(w.rep, K, ~0ull, st));
    CAT_TRY(launch_count_rep(assignments, N, K, w.counts, w.rep, st));
    CAT_TRY(step_stats(lq, fp, dt, assignments, N, D, K, w.counts, w.rep, centroids, w, gamma, beta, st));
    if (counts) CAT_TRY(launch_copy_words(w.counts, counts, K, st));
    return CAT_OK;
}

static cat_status fit_impl(const char* who, const void* lq, const void* fp, int64_t N, int64_t D, int32_t K,
                           int32_t iters, uint64_t seed, cat_dtype dt, const float* init_centroids, float* centroids,
                           float* gamma, float* beta, int32_t* assignments, int32_t* counts, double* inertia,
                           int32_t* skipped, void* workspace, size_t workspace_bytes, void* hip_stream,
                           bool with_bounds = false, int32_t* evaluated = nullptr) {
    CAT_TRY(check_shape(who, N, D, K, dt));
    if (iters < 0) return set_error(CAT_ERR_INVALID_ARG, "%s: iters = %d is negative", who, (int)iters);
    CAT_TRY(check_ptr(who, "lq", lq, 16));
    CAT_TRY(check_ptr(who, "fp", fp, 16));
    if (init_centroids) CAT_TRY(check_ptr(who, "init_centroids", init_centroids, 16));
    CAT_TRY(check_ptr(who, "centroids", centroids, 16));
    CAT_TRY(check_ptr(who, "gamma", gamma, 16));
    CAT_TRY(check_ptr(who, "beta", beta, 16));
    CAT_TRY(check_ptr(who, "assignments", assignments, 4));
    if (inertia) CAT_TRY(check_ptr(who, "inertia", inertia, 8));
    FitWs w = carve_fit(workspace, N, D, K, dt);
    BoundsWs bw;
    size_t need = w.bytes;
    if (with_bounds) {
        bw = bounds_carve(workspace ? (char*)workspace + align256(w.bytes) : nullptr, N, D, K, iters);
        bw.evaluated = evaluated;
        need = align256(w.bytes) + bw.bytes;
    }
    // rows that are not whole 16-byte groups: the clustering runs on a zero-padded copy (the scratch sizes of the fits
    // include it; the entry points that size their scratch from the pieces do not come through here)
    const bool padded = fit_runs_padded(N, D, K, dt, iters);
    PadWs pw;
    if (padded) {
        pw = carve_pad(workspace ? (char*)workspace + align256(need) : nullptr, N, D, K, dt, iters, with_bounds);
        need = align256(need) + pw.bytes;
    }
    CAT_TRY(check_ws(who, workspace, workspace_bytes, need));
    hipStream_t st = (hipStream_t)hip_stream;
    if (padded) {
        const int64_t Dp = pw.Dp;
        FitWs wp = carve_fit(pw.fit, N, Dp, K, dt);
        BoundsWs bp;
        if (with_bounds) {
            bp = bounds_carve(pw.bounds, N, Dp, K, iters);
            bp.evaluated = evaluated;
        }
        CAT_TRY(launch_pad_rows(lq, dt, N, D, Dp, pw.lq, st));
        if (init_centroids) CAT_TRY(launch_pad_rows(init_centroids, CAT_F32, K, D, Dp, pw.init, st));
        CAT_TRY(run_lloyd(pw.lq, dt, N, Dp, K, iters, seed, init_centroids ? pw.init : nullptr, pw.cent, assignments, inertia,
                          wp, st, skipped, with_bounds ? &bp : nullptr));
        CAT_TRY(launch_pad_rows(pw.cent, CAT_F32, K, Dp, D, centroids, st));
        w = wp;  // counts and first rows of the clusters are there; its arrays are at least as large
    } else {
        CAT_TRY(run_lloyd(lq, dt, N, D, K, iters, seed, init_centroids, centroids, assignments, inertia, w, st, skipped,
                          with_bounds ? &bw : nullptr));
    }
    // affine fit on that partition, shifted by the centroids
    CAT_TRY(step_stats(lq, fp, dt, assignments, N, D, K, w.counts, w.rep, centroids, w, gamma, beta, st));
    if (counts) CAT_TRY(launch_copy_words(w.counts, counts, K, st));
    return CAT_OK;
}

cat_status cat_fit(const void* lq, const void* fp, int64_t N, int64_t D, int32_t K, int32_t iters, uint64_t seed,
                   cat_dtype dt, const float* init_centroids, float* centroids, float* gamma, float* beta,
                   int32_t* assignments, int32_t* counts, double* inertia, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
    return fit_impl("cat_fit", lq, fp, N, D, K, iters, seed, dt, init_centroids, centroids, gamma, beta, assignments,
                    counts, inertia, nullptr, workspace, workspace_bytes, hip_stream);
}

cat_status cat_fit_early_stop(const void* lq, const void* fp, int64_t N, int64_t D, int32_t K, int32_t iters,
                              uint64_t seed, cat_dtype dt, const float* init_centroids, float* centroids, float* gamma,
                              float* beta, int32_t* assignments, int32_t* counts, double* inertia,
                              int32_t* passes_skipped, void* workspace, size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_ptr("cat_fit_early_stop", "passes_skipped", passes_skipped, 4));
    return fit_impl("cat_fit_early_stop", lq, fp, N, D, K, iters, seed, dt, init_centroids, centroids, gamma, beta,
                    assignments, counts, inertia, passes_skipped, workspace, workspace_bytes, hip_stream);
}

size_t cat_fit_bounds_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt) || iters < 0) return 0;
    size_t b = align256(carve_fit(nullptr, N, D, K, dt).bytes) + bounds_workspace_bytes(N, D, K, iters);
    if (pad_applies(N, D, K, dt)) b = align256(b) + carve_pad(nullptr, N, D, K, dt, iters, true).bytes;
    return b;
}

cat_status cat_fit_bounds(const void* lq, const void* fp, int64_t N, int64_t D, int32_t K, int32_t iters, uint64_t seed,
                          cat_dtype dt, const float* init_centroids, float* centroids, float* gamma, float* beta,
                          int32_t* assignments, int32_t* counts, double* inertia, int32_t* rows_evaluated, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
    if (rows_evaluated) CAT_TRY(check_ptr("cat_fit_bounds", "rows_evaluated", rows_evaluated, 4));
    if (N >= ((int64_t)1 << 31))
        return set_error(CAT_ERR_UNSUPPORTED, "cat_fit_bounds: N = %lld does not fit the 32-bit row numbers of its lists", (long long)N);
    const bool fused = (tile_supports(TILE_LLOYD, N, D, K, dt) && g_path.load() != CAT_PATH_STREAM) || fit_runs_padded(N, D, K, dt, iters);
    cat_status s = fit_impl("cat_fit_bounds", lq, fp, N, D, K, iters, seed, dt, init_centroids, centroids, gamma, beta,
                            assignments, counts, inertia, nullptr, workspace, workspace_bytes, hip_stream, true, rows_evaluated);
    if (s != CAT_OK) return s;
    // the kernels outside the matrix-core family keep no bounds: every pass evaluates every row
    if (!fused && rows_evaluated) return launch_fill_i32(rows_evaluated, (int64_t)iters + 1, (int32_t)N, (hipStream_t)hip_stream);
    return CAT_OK;
}

// ---- several runs of the clustering, the one with the lowest final objective kept ---------------------
struct RestartWs {
    void* fit;           // cat_fit scratch
    void* pp;            // cat_init_kmeanspp scratch
    float* init;         // K x D   seeded centroids of the run
    float* cent;         // K x D   centroids of the run
    int32_t* assign;     // N       assignments of the run
    double* inertia;     // iters + 1 objective values of the run
    double* best;        // lowest final objective so far
    int32_t* state;      // [0] the run just finished is the best so far, [1] its index
    void* pad;           // scratch of the runs on a zero-padded copy of the rows (only for the shapes that use one)
    size_t fit_bytes, pp_bytes, bytes;
};
static RestartWs carve_restarts(void* base, int64_t N, int64_t D, int32_t K, int32_t iters, cat_dtype dt) {
    RestartWs w;
    w.fit_bytes = carve_fit(nullptr, N, D, K, dt).bytes;
    w.pp_bytes = cat_init_kmeanspp_workspace_bytes(N, K);
    char* b = (char*)base;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* ptr = b + off;
        off += align256(bytes);
        return ptr;
    };
    w.fit = take(w.fit_bytes);
    w.pp = take(w.pp_bytes);
    w.init = (float*)take((size_t)K * (size_t)D * sizeof(float));
    w.cent = (float*)take((size_t)K * (size_t)D * sizeof(float));
    w.assign = (int32_t*)take((size_t)N * sizeof(int32_t));
    w.inertia = (double*)take(((size_t)(iters < 0 ? 0 : iters) + 1) * sizeof(double));
    w.best = (double*)take(sizeof(double));
    w.state = (int32_t*)take(2 * sizeof(int32_t));
    w.pad = pad_applies(N, D, K, dt) ? take(carve_pad(nullptr, N, D, K, dt, iters, false).bytes) : nullptr;
    w.bytes = off;
    return w;
}

size_t cat_fit_restarts_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt) || iters < 0) return 0;
    return carve_restarts(nullptr, N, D, K, iters, dt).bytes;
}

cat_status cat_fit_restarts(const void* lq, const void* fp, int64_t N, int64_t D, int32_t K, int32_t iters, uint64_t seed,
                            int32_t restarts, cat_seeding seeding, cat_dtype dt, float* centroids, float* gamma, float* beta,
                            int32_t* assignments, int32_t* counts, double* inertia, int32_t* best_run, double* final_inertia,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_shape("cat_fit_restarts", N, D, K, dt));
    if (iters < 0) return set_error(CAT_ERR_INVALID_ARG, "cat_fit_restarts: iters = %d is negative", (int)iters);
    if (restarts < 1 || restarts > CAT_MAX_RESTARTS)
        return set_error(CAT_ERR_INVALID_ARG, "cat_fit_restarts: need 1 <= restarts <= %d (got %d)", CAT_MAX_RESTARTS, (int)restarts);
    if (seeding != CAT_SEED_ROWS && seeding != CAT_SEED_KMEANSPP)
        return set_error(CAT_ERR_INVALID_ARG, "cat_fit_restarts: unknown seeding %d", (int)seeding);
    CAT_TRY(check_ptr("cat_fit_restarts", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_fit_restarts", "fp", fp, 16));
    CAT_TRY(check_ptr("cat_fit_restarts", "centroids", centroids, 16));
    CAT_TRY(check_ptr("cat_fit_restarts", "gamma", gamma, 16));
    CAT_TRY(check_ptr("cat_fit_restarts", "beta", beta, 16));
    CAT_TRY(check_ptr("cat_fit_restarts", "assignments", assignments, 4));
    if (inertia) CAT_TRY(check_ptr("cat_fit_restarts", "inertia", inertia, 8));
    if (final_inertia) CAT_TRY(check_ptr("cat_fit_restarts", "final_inertia", final_inertia, 8));
    RestartWs w = carve_restarts(workspace, N, D, K, iters, dt);
    CAT_TRY(check_ws("cat_fit_restarts", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    FitWs fw = carve_fit(w.fit, N, D, K, dt);
    const size_t KD = (size_t)K * (size_t)D;
    // as in cat_fit: rows that are not whole 16-byte groups are padded once, every run clusters the copy
    const bool padded = fit_runs_padded(N, D, K, dt, iters);
    PadWs pw;
    FitWs wp;
    if (padded) {
        pw = carve_pad(w.pad, N, D, K, dt, iters, false);
        wp = carve_fit(pw.fit, N, pw.Dp, K, dt);
        CAT_TRY(launch_pad_rows(lq, dt, N, D, pw.Dp, pw.lq, st));
    }
    for (int32_t r = 0; r < restarts; r++) {
        const uint64_t seed_r = seed + (uint64_t)r;
        const float* init = nullptr;
        if (seeding == CAT_SEED_KMEANSPP) {
            CAT_TRY(cat_init_kmeanspp(lq, N, D, K, seed_r, dt, w.init, nullptr, w.pp, w.pp_bytes, hip_stream));
            init = w.init;
        }
        if (padded) {
            if (init) CAT_TRY(launch_pad_rows(init, CAT_F32, K, D, pw.Dp, pw.init, st));
            CAT_TRY(run_lloyd(pw.lq, dt, N, pw.Dp, K, iters, seed_r, init ? pw.init : nullptr, pw.cent, w.assign, w.inertia, wp, st));
            CAT_TRY(launch_pad_rows(pw.cent, CAT_F32, K, pw.Dp, D, w.cent, st));
        } else {
            CAT_TRY(run_lloyd(lq, dt, N, D, K, iters, seed_r, init, w.cent, w.assign, w.inertia, fw, st));
        }
        CAT_TRY(launch_keep_best(w.inertia + iters, w.best, w.state, r, final_inertia, st));
        CAT_TRY(launch_copy_words_if(w.state, w.cent, centroids, (int64_t)KD, st));
        CAT_TRY(launch_copy_words_if(w.state, w.assign, assignments, N, st));
        if (inertia) CAT_TRY(launch_copy_words_if(w.state, w.inertia, inertia, 2 * ((int64_t)iters + 1), st));
    }
    // the kept partition: counts and first rows again (the scratch holds those of the last run), then the affine fit
    CAT_TRY(launch_fill_zero(fw.counts, (size_t)K * sizeof(int32_t), st));
    CAT_TRY(launch_fill_u64(fw.rep, K, ~0ull, st));
    CAT_TRY(launch_count_rep(assignments, N, K, fw.counts, fw.rep, st));
    CAT_TRY(step_stats(lq, fp, dt, assignments, N, D, K, fw.counts, fw.rep, centroids, fw, gamma, beta, st));
    if (counts) CAT_TRY(launch_copy_words(fw.counts, counts, K, st));
    if (best_run) CAT_TRY(launch_copy_words(w.state + 1, best_run, 1, st));
    return CAT_OK;
}

// ---- fits for a grid of cluster counts that share the reads of the rows --------------------------------
// Consecutive entries of Ks whose 16-cluster tiles fit one launch of the tile kernel together form a group and run
// their Lloyd loops side by side (tile_lloyd_multi); an entry the tile kernels cannot take, or one left alone, runs
// the ordinary loop.  The plan depends on the arguments only, so the workspace query and the call agree.
// Tiles per group; 0: chosen from the shape.  Measured on the paper's grid of eleven counts (1 .. 256): groups pay where a
// pass is bound by the read of the rows (counts up to about 32: 0.6 of the time of separate fits).  Rows of more than
// 1 KB make a pass of more than 4 cluster tiles contraction-bound, where sharing the read gains nothing and the larger
// kernel costs (65536 x 1000: the counts 48 and 64 together 6.7 ms, apart 5.6 ms), so groups stop at 4 tiles there and
// at 8 for shorter rows (65536 x 52: the grid in 12.1 ms with 8, 12.9 ms with 4); 16-tile instances spill registers.
static std::atomic<int> g_multi_tiles{0};  // cat_debug_multi_group_tiles

struct MultiGroup {
    int first = 0, count = 0;
    MultiSets ms;
};
static std::vector<MultiGroup> plan_multi(int64_t N, int64_t D, const int32_t* Ks, int32_t nK, cat_dtype dt) {
    std::vector<MultiGroup> groups;
    int cap = g_multi_tiles.load();
    if (cap == 0) cap = D * (dt == CAT_BF16 ? 2 : 4) <= 1024 ? 8 : 4;
    const bool tiles_allowed = g_path.load() != CAT_PATH_STREAM;
    while (cap > 1 && !tile_multi_supports(N, D, 16 * cap, 1, dt)) cap /= 2;
    if (!tiles_allowed || !tile_multi_supports(N, D, 16 * cap, 1, dt)) cap = 0;
    MultiGroup cur;
    auto flush = [&]() {
        if (cur.count) groups.push_back(cur);
        cur = MultiGroup();
    };
    for (int i = 0; i < nK; i++) {
        const int tiles = (Ks[i] + 15) / 16;
        const bool fits = cap > 0 && tiles <= cap;
        if (!fits) {
            flush();
            cur.first = i;
            cur.count = 1;
            cur.ms.nsets = 0;  // marks a set that runs the ordinary loop
            flush();
            continue;
        }
        if (cur.count && (cur.ms.t0[cur.ms.nsets] + tiles > cap || cur.ms.nsets == 16 ||
                          N * (int64_t)(cur.ms.nsets + 1) >= ((int64_t)1 << 32)))
            flush();
        if (!cur.count) cur.first = i;
        cur.ms.k[cur.ms.nsets] = Ks[i];
        cur.ms.t0[cur.ms.nsets + 1] = cur.ms.t0[cur.ms.nsets] + tiles;
        cur.ms.nsets++;
        cur.count++;
    }
    flush();
    for (auto& g : groups)
        if (g.count == 1) g.ms.nsets = 0;  // alone: the ordinary loop (no table of 16 assignments per row)
    return groups;
}

struct MultiWs {
    void* fit;            // cat_fit scratch, large enough for every K of the call (ordinary loops, the affine fits)
    float* cent;          // slots x D   centroids of a group, by slot
    double* sums;         // 2 x slots x D
    int32_t* assign16;    // N x 16
    int32_t* counts;      // slots
    unsigned long long* rep;  // slots
    double* inertia16;    // (iters + 1) x 16
    int32_t* column;      // N
    void* lqpad;          // N x D rows padded with zero channels, and K x D centroids of a fit on them (only where
    float* centpad;       //   the loops run on the padded copy)
    TileWs tile;
    LloydWs lloyd;
    size_t fit_bytes, bytes;
};
// D: the row length the Lloyd loops see; Dorig < D where they run on a zero-padded copy of the rows
static MultiWs carve_multi(void* base, int64_t N, int64_t D, const int32_t* Ks, int32_t nK, int32_t slots, int32_t nsets,
                           int32_t iters, cat_dtype dt, int64_t Dorig) {
    MultiWs w = {};
    w.fit_bytes = 0;  // the scratch of one fit is not monotone in K (the tile kernels take some K and not others)
    int32_t Kmax = 1;
    for (int i = 0; i < nK; i++) {
        size_t b = carve_fit(nullptr, N, D, Ks[i], dt).bytes;
        if (Dorig != D) {
            const size_t bo = carve_fit(nullptr, N, Dorig, Ks[i], dt).bytes;
            b = bo > b ? bo : b;
        }
        w.fit_bytes = b > w.fit_bytes ? b : w.fit_bytes;
        Kmax = Ks[i] > Kmax ? Ks[i] : Kmax;
    }
    Carver c(base);
    w.fit = c.take<char>(w.fit_bytes);
    if (Dorig != D) {
        w.lqpad = c.take<char>((size_t)N * (size_t)D * (dt == CAT_BF16 ? 2 : 4));
        w.centpad = c.take<float>((size_t)Kmax * (size_t)D);
    }
    if (slots > 0) {
        const size_t SD = (size_t)slots * (size_t)D;
        w.cent = c.take<float>(SD);
        w.sums = c.take<double>(2 * SD);
        w.assign16 = c.take<int32_t>((size_t)N * 16);
        w.counts = c.take<int32_t>(slots);
        w.rep = c.take<unsigned long long>(slots);
        w.inertia16 = c.take<double>(((size_t)iters + 1) * 16);
        w.column = c.take<int32_t>((size_t)N);
        const size_t tb = tile_workspace_bytes(D, slots, dt);
        w.tile = tile_carve(base ? (void*)(c.base + c.off) : nullptr, D, slots, dt);
        c.off += align256(tb);
        w.lloyd = lloyd_carve(base ? (void*)(c.base + c.off) : nullptr, N * (int64_t)nsets, D, slots);
        c.off += align256(w.lloyd.bytes);
    }
    w.bytes = c.off;
    return w;
}

static cat_status check_multi(const char* who, int64_t N, int64_t D, const int32_t* Ks, int32_t nK, int32_t iters, cat_dtype dt) {
    if (!Ks || nK < 1 || nK > CAT_MAX_MULTI_K)
        return set_error(CAT_ERR_INVALID_ARG, "%s: need a host array of 1 .. %d cluster counts (got %d)", who, CAT_MAX_MULTI_K, (int)nK);
    if (iters < 0) return set_error(CAT_ERR_INVALID_ARG, "%s: iters = %d is negative", who, (int)iters);
    for (int i = 0; i < nK; i++) CAT_TRY(check_shape(who, N, D, Ks[i], dt));
    return CAT_OK;
}

static void multi_extent(const std::vector<MultiGroup>& groups, const int32_t* Ks, int32_t nK, int32_t& Kmax, int32_t& slots,
                         int32_t& nsets) {
    Kmax = 1, slots = 0, nsets = 0;
    for (int i = 0; i < nK; i++) Kmax = Ks[i] > Kmax ? Ks[i] : Kmax;
    for (const auto& g : groups) {
        if (!g.ms.nsets) continue;
        slots = 16 * g.ms.t0[g.ms.nsets] > slots ? 16 * g.ms.t0[g.ms.nsets] : slots;
        nsets = g.ms.nsets > nsets ? g.ms.nsets : nsets;
    }
}

// The same rule as for a single fit: rows that are not whole 16-byte groups are copied once, padded with zero channels,
// and every cluster count the matrix-core kernels take at the padded length clusters on the copy.
static bool multi_runs_padded(int64_t N, int64_t D, const int32_t* Ks, int32_t nK, cat_dtype dt, int32_t iters) {
    for (int i = 0; i < nK; i++)
        if (fit_runs_padded(N, D, Ks[i], dt, iters)) return true;
    return false;
}

cat_status cat_debug_multi_group_tiles(int tiles) {
    if (tiles != 0 && tiles != 1 && tiles != 2 && tiles != 4 && tiles != 8)
        return set_error(CAT_ERR_INVALID_ARG, "cat_debug_multi_group_tiles: %d is not 0, 1, 2, 4 or 8", tiles);
    g_multi_tiles.store(tiles);
    return CAT_OK;
}

size_t cat_fit_multi_k_workspace_bytes(int64_t N, int64_t D, const int32_t* Ks, int32_t nK, int32_t iters, cat_dtype dt) {
    if (!Ks || nK < 1 || nK > CAT_MAX_MULTI_K || iters < 0) return 0;
    for (int i = 0; i < nK; i++)
        if (!shape_ok(N, D, Ks[i], dt)) return 0;
    int32_t Kmax, slots, nsets;
    const int64_t Dl = multi_runs_padded(N, D, Ks, nK, dt, iters) ? padded_dim(D, dt) : D;
    multi_extent(plan_multi(N, Dl, Ks, nK, dt), Ks, nK, Kmax, slots, nsets);
    return carve_multi(nullptr, N, Dl, Ks, nK, slots, nsets, iters, dt, D).bytes;
}

cat_status cat_fit_multi_k(const void* lq, const void* fp, int64_t N, int64_t D, const int32_t* Ks, int32_t nK, int32_t iters,
                           uint64_t seed, cat_dtype dt, float* centroids, float* gamma, float* beta, int32_t* assignments,
                           int32_t* counts, double* inertia, void* workspace, size_t workspace_bytes, void* hip_stream) {
    const char* who = "cat_fit_multi_k";
    CAT_TRY(check_multi(who, N, D, Ks, nK, iters, dt));
    CAT_TRY(check_ptr(who, "lq", lq, 16));
    CAT_TRY(check_ptr(who, "fp", fp, 16));
    CAT_TRY(check_ptr(who, "centroids", centroids, 16));
    CAT_TRY(check_ptr(who, "gamma", gamma, 16));
    CAT_TRY(check_ptr(who, "beta", beta, 16));
    CAT_TRY(check_ptr(who, "assignments", assignments, 4));
    if (inertia) CAT_TRY(check_ptr(who, "inertia", inertia, 8));
    const bool padded = multi_runs_padded(N, D, Ks, nK, dt, iters);
    const int64_t Dl = padded ? padded_dim(D, dt) : D;  // the row length the Lloyd loops see
    const std::vector<MultiGroup> groups = plan_multi(N, Dl, Ks, nK, dt);
    int32_t Kmax, slots, nsets;
    multi_extent(groups, Ks, nK, Kmax, slots, nsets);
    MultiWs w = carve_multi(workspace, N, Dl, Ks, nK, slots, nsets, iters, dt, D);
    CAT_TRY(check_ws(who, workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    if (padded) CAT_TRY(launch_pad_rows(lq, dt, N, D, Dl, w.lqpad, st));
    const void* lql = padded ? w.lqpad : lq;
    std::vector<int64_t> row0(nK + 1, 0);  // first row of set i in centroids / gamma / beta / counts
    for (int i = 0; i < nK; i++) row0[i + 1] = row0[i] + Ks[i];
    const int64_t nin = (int64_t)iters + 1;
    for (const auto& g : groups) {
        if (!g.ms.nsets) {  // the ordinary fit
            const int i = g.first;
            const int32_t K = Ks[i];
            float* cent_i = centroids + row0[i] * D;
            int32_t* asg_i = assignments + (int64_t)i * N;
            double* in_i = inertia ? inertia + i * nin : nullptr;
            // (a count the matrix-core kernels do not take at the padded length either: the original rows, as cat_fit does)
            const bool on_copy = padded && tile_supports(TILE_LLOYD, N, Dl, K, dt);
            FitWs fw = carve_fit(w.fit, N, on_copy ? Dl : D, K, dt);
            if (on_copy) {
                CAT_TRY(run_lloyd(w.lqpad, dt, N, Dl, K, iters, seed, nullptr, w.centpad, asg_i, in_i, fw, st));
                CAT_TRY(launch_pad_rows(w.centpad, CAT_F32, K, Dl, D, cent_i, st));
            } else {
                CAT_TRY(run_lloyd(lq, dt, N, D, K, iters, seed, nullptr, cent_i, asg_i, in_i, fw, st));
            }
            CAT_TRY(step_stats(lq, fp, dt, asg_i, N, D, K, fw.counts, fw.rep, cent_i, fw, gamma + row0[i] * D,
                               beta + row0[i] * D, st));
            if (counts) CAT_TRY(launch_copy_words(fw.counts, counts + row0[i], K, st));
            continue;
        }
        const MultiSets& ms = g.ms;
        const int32_t gslots = 16 * ms.t0[ms.nsets];
        // seeded rows of every set into its slots; the other slots stay zero rows with zero counts
        CAT_TRY(launch_fill_zero(w.cent, (size_t)gslots * Dl * sizeof(float), st));
        FitWs fw = carve_fit(w.fit, N, Dl, Kmax, dt);
        for (int j = 0; j < ms.nsets; j++) {
            CAT_TRY(launch_init_indices(N, ms.k[j], seed, fw.idx, st));
            CAT_TRY(launch_gather_rows(lql, dt, Dl, ms.k[j], fw.idx, w.cent + (size_t)16 * ms.t0[j] * Dl, st));
        }
        LloydWs lw = w.lloyd;
        lw.sort_ws = fw.sort;
        CAT_TRY(tile_lloyd_multi(lql, dt, N, Dl, ms, iters, w.cent, w.sums, w.assign16, w.counts, inertia ? w.inertia16 : nullptr,
                                 w.rep, w.column, w.tile, lw, st));
        for (int j = 0; j < ms.nsets; j++) {
            const int i = g.first + j;
            const int32_t K = ms.k[j], slot0 = 16 * ms.t0[j];
            float* cent_i = centroids + row0[i] * D;
            int32_t* asg_i = assignments + (int64_t)i * N;
            CAT_TRY(launch_multi_column(w.assign16, N, j, slot0, asg_i, st));
            if (padded)
                CAT_TRY(launch_pad_rows(w.cent + (size_t)slot0 * Dl, CAT_F32, K, Dl, D, cent_i, st));
            else
                CAT_TRY(launch_copy_words(w.cent + (size_t)slot0 * D, cent_i, (int64_t)K * D, st));
            FitWs fk = carve_fit(w.fit, N, D, K, dt);
            CAT_TRY(step_stats(lq, fp, dt, asg_i, N, D, K, w.counts + slot0, w.rep + slot0, cent_i, fk, gamma + row0[i] * D,
                               beta + row0[i] * D, st));
            if (counts) CAT_TRY(launch_copy_words(w.counts + slot0, counts + row0[i], K, st));
            if (inertia)
                CAT_TRY(launch_copy_cols((const float*)(w.inertia16 + j), nin, 32, (float*)(inertia + i * nin), 2, 2, st));
        }
    }
    return CAT_OK;
}

// Argument checks and launches of CAT Inferencing over a scratch buffer of `workspace_bytes` bytes at `workspace`
// (the caller's for cat_apply, the library's own for cat_apply_static).
static cat_status apply_impl(const char* who, const void* lq, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                             const float* centroids, const float* gamma, const float* beta, float alpha, void* corrected,
                             int32_t* assignments, void* workspace, size_t workspace_bytes, hipStream_t st) {
    CAT_TRY(check_shape(who, N, D, K, dt));
    CAT_TRY(check_ptr(who, "lq", lq, 16));
    CAT_TRY(check_ptr(who, "centroids", centroids, 16));
    CAT_TRY(check_ptr(who, "gamma", gamma, 16));
    CAT_TRY(check_ptr(who, "beta", beta, 16));
    CAT_TRY(check_ptr(who, "corrected", corrected, 16));
    if (corrected == lq) return set_error(CAT_ERR_INVALID_ARG, "%s: corrected may not alias lq", who);
    if (!std::isfinite(alpha)) return set_error(CAT_ERR_INVALID_ARG, "%s: alpha is not finite", who);
    // (a workspace of the size without the scratch of the split ranking is accepted: cat_apply_static has no more)
    ApplyWs w = carve_apply(workspace, D, K, dt, N);
    if (w.split && workspace && workspace_bytes < w.bytes) w = carve_apply(workspace, D, K, dt);
    CAT_TRY(check_ws(who, workspace, workspace_bytes, w.bytes));
    const float* g = gamma;
    const float* b = beta;
    if (alpha != 1.0f) {
        CAT_TRY(launch_fold_alpha(gamma, beta, alpha, w.g_eff, w.b_eff, (int64_t)K * D, st));
        g = w.g_eff;
        b = w.b_eff;
    }
    const int path = g_path.load();
    const bool tile_ok = tile_supports(TILE_APPLY, N, D, K, dt);
    if (path == CAT_PATH_TILE && !tile_ok)
        return set_error(CAT_ERR_UNSUPPORTED, "tile path forced but D=%lld K=%d dt=%d does not fit it", (long long)D,
                         (int)K, (int)dt);
    // two fused kernels: the row-tile kernel reads every row once (its instances cover the shapes whose centroid
    // operand the 8 waves of a workgroup can hold in registers), the tile kernel takes the rest
    const int which = g_apply_kernel.load();
    const bool rowtile_ok = infer_supported(N, D, K, dt);
    if (which == 2 && !rowtile_ok)
        return set_error(CAT_ERR_UNSUPPORTED, "row-tile inference kernel forced but D=%lld K=%d dt=%d does not fit it",
                         (long long)D, (int)K, (int)dt);
    if (rowtile_ok && path != CAT_PATH_STREAM && which != 1)
        return infer_apply(lq, dt, N, D, K, centroids, g, b, corrected, assignments, w.tile, st);
    if (tile_ok && path != CAT_PATH_STREAM && w.split && which == 0) {
        // more than 128 clusters: ranked by two launches of 8 cluster tiles, then mapped by the labels (the fused
        // 16-tile kernel ranks with the one-part operand and re-ranks most rows: several times slower)
        int32_t* labels = assignments ? assignments : w.labels;
        CAT_TRY(tile_assign_split(lq, dt, N, D, K, centroids, labels, nullptr, nullptr, nullptr, w.tile, w.split, st));
        return launch_affine_by_labels(lq, dt, labels, N, D, g, b, corrected, false, st);
    }
    if (tile_ok && path != CAT_PATH_STREAM)
        return tile_assign(lq, dt, N, D, K, centroids, assignments, nullptr, nullptr, nullptr, g, b, corrected, w.tile,
                           st);
    if (path != CAT_PATH_STREAM)
        return launch_assign_lds(lq, dt, N, D, K, centroids, assignments, nullptr, nullptr, nullptr, g, b, corrected, st);
    return launch_assign_stream(lq, dt, N, D, K, centroids, assignments, nullptr, nullptr, nullptr, g, b, corrected,
                                st);
}

cat_status cat_apply(const void* lq, int64_t N, int64_t D, int32_t K, cat_dtype dt, const float* centroids,
                     const float* gamma, const float* beta, float alpha, void* corrected, int32_t* assignments,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    return apply_impl("cat_apply", lq, N, D, K, dt, centroids, gamma, beta, alpha, corrected, assignments, workspace,
                      workspace_bytes, (hipStream_t)hip_stream);
}

// ---- low-precision deployment: parameters stored as bfloat16, corrected rows optionally written as bfloat16 ----
struct ApplyLpWs {
    float* cent;      // K x D   the stored parameters as fp32 working arrays (alpha folded into g, b)
    float* g;
    float* b;
    int32_t* labels;  // N       for the shapes that assign first and map afterwards
    void* apply;      // cat_apply scratch
    size_t apply_bytes, bytes;
};
static ApplyLpWs carve_apply_lp(void* base, int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    Carver c(base);
    ApplyLpWs w;
    const size_t KD = (size_t)K * (size_t)D;
    w.cent = c.take<float>(KD);
    w.g = c.take<float>(KD);
    w.b = c.take<float>(KD);
    w.labels = c.take<int32_t>((size_t)N);
    w.apply_bytes = carve_apply(nullptr, D, K, dt, N).bytes;
    w.apply = c.take<char>(w.apply_bytes);
    w.bytes = c.off;
    return w;
}

cat_status cat_params_to_bf16(const float* src, int64_t n, uint16_t* dst, void* hip_stream) {
    CAT_TRY(check_ptr("cat_params_to_bf16", "src", src, 4));
    CAT_TRY(check_ptr("cat_params_to_bf16", "dst", dst, 2));
    if (n < 0) return set_error(CAT_ERR_INVALID_ARG, "cat_params_to_bf16: n = %lld is negative", (long long)n);
    if (n == 0) return CAT_OK;
    return launch_to_bf16(src, n, dst, (hipStream_t)hip_stream);
}

size_t cat_apply_lp_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt)) return 0;
    return carve_apply_lp(nullptr, N, D, K, dt).bytes;
}

cat_status cat_apply_lp(const void* lq, int64_t N, int64_t D, int32_t K, cat_dtype dt, const uint16_t* centroids,
                        const uint16_t* gamma, const uint16_t* beta, float alpha, cat_dtype out_dt, void* corrected,
                        int32_t* assignments, void* workspace, size_t workspace_bytes, void* hip_stream) {
    const char* who = "cat_apply_lp";
    CAT_TRY(check_shape(who, N, D, K, dt));
    if (out_dt != CAT_F32 && out_dt != CAT_BF16) return set_error(CAT_ERR_INVALID_ARG, "%s: unknown out_dt %d", who, (int)out_dt);
    if (dt == CAT_BF16 && out_dt != CAT_BF16)
        return set_error(CAT_ERR_INVALID_ARG, "%s: bf16 rows are corrected into bf16 rows (out_dt = CAT_BF16)", who);
    CAT_TRY(check_ptr(who, "lq", lq, 16));
    CAT_TRY(check_ptr(who, "centroids", centroids, 2));
    CAT_TRY(check_ptr(who, "gamma", gamma, 2));
    CAT_TRY(check_ptr(who, "beta", beta, 2));
    CAT_TRY(check_ptr(who, "corrected", corrected, 16));
    if (corrected == lq) return set_error(CAT_ERR_INVALID_ARG, "%s: corrected may not alias lq", who);
    if (!std::isfinite(alpha)) return set_error(CAT_ERR_INVALID_ARG, "%s: alpha is not finite", who);
    ApplyLpWs w = carve_apply_lp(workspace, N, D, K, dt);
    CAT_TRY(check_ws(who, workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    CAT_TRY(launch_expand_params(centroids, gamma, beta, alpha, (int64_t)K * D, w.cent, w.g, w.b, st));
    if (out_dt == dt)  // the ordinary inference on the expanded parameters (alpha is folded in already)
        return apply_impl(who, lq, N, D, K, dt, w.cent, w.g, w.b, 1.0f, corrected, assignments, w.apply, w.apply_bytes, st);
    // fp32 rows, bfloat16 out: the row-tile kernel writes the narrower rows itself; shapes it has no instance for
    // assign first and map by the labels afterwards (a second read of the rows)
    ApplyWs aw = carve_apply(w.apply, D, K, dt, N);
    const int path = g_path.load();
    if (infer_supported(N, D, K, dt) && path != CAT_PATH_STREAM && g_apply_kernel.load() != 1)
        return infer_apply(lq, dt, N, D, K, w.cent, w.g, w.b, corrected, assignments, aw.tile, st, true);
    int32_t* labels = assignments ? assignments : w.labels;
    CAT_TRY(step_assign(lq, dt, N, D, K, w.cent, labels, nullptr, nullptr, nullptr, aw.tile, st, aw.split));
    return launch_affine_by_labels(lq, dt, labels, N, D, w.g, w.b, corrected, true, st);
}

// ---- cat_apply for callers that cannot allocate: the scratch memory is a device array of the library ----
// One copy of the array exists on every GPU the library runs on, at an address of its own, and stays there until the
// process ends.  The name of the array is a host-side stand-in, not a device address: host code only ever uses the
// per-device address that hipGetSymbolAddress returns (asked once per device, with that device current).
static __device__ __align__(256) unsigned char scratch[CAT_APPLY_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static cat_status static_scratch(void** out) {
    int dev = 0;
    CAT_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return set_error(CAT_ERR_DEVICE, "cat_apply_static: device ordinal %d out of range", dev);
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // two threads racing here ask twice and store the same address
        CAT_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return set_error(CAT_ERR_DEVICE, "cat_apply_static: the scratch array has no address on device %d", dev);
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return CAT_OK;
}

size_t cat_apply_static_max_workspace_bytes(void) { return CAT_APPLY_STATIC_SCRATCH_BYTES; }

cat_status cat_apply_static(const void* lq, int64_t N, int64_t D, int32_t K, cat_dtype dt, const float* centroids,
                            const float* gamma, const float* beta, float alpha, void* corrected, int32_t* assignments,
                            void* hip_stream) {
    CAT_TRY(check_shape("cat_apply_static", N, D, K, dt));
    const size_t need = carve_apply(nullptr, D, K, dt).bytes;
    if (need > (size_t)CAT_APPLY_STATIC_SCRATCH_BYTES)
        return set_error(CAT_ERR_UNSUPPORTED,
                         "cat_apply_static: D=%lld K=%d needs %zu bytes of scratch, the built-in array holds %zu; use "
                         "cat_apply with a workspace",
                         (long long)D, (int)K, need, (size_t)CAT_APPLY_STATIC_SCRATCH_BYTES);
    void* ptr = nullptr;
    CAT_TRY(static_scratch(&ptr));
    // nothing in the scratch has to start at zero: the fold of alpha and the centroid preparation overwrite every
    // byte the inference pass reads
    return apply_impl("cat_apply_static", lq, N, D, K, dt, centroids, gamma, beta, alpha, corrected, assignments, ptr,
                      (size_t)CAT_APPLY_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream);
}


// ---- Algorithms 1 and 2 with the PCA front-end, as single calls -----------------------------------
// The scores are kept with rows of pad4(p) floats, the padding columns zero (they add nothing to a distance):
// rows then keep the 16-byte alignment the tile kernels need, whatever p is.
static inline int32_t pad4(int32_t p) { return (p + 3) & ~3; }
struct PcaFitWs {
    void* pca;      // cat_pca_fit scratch
    float* z;       // N x pad4(p) scores
    float* cz;      // K x pad4(p) centroids in score space
    void* lloyd;    // cat_fit scratch for (N, pad4(p), K, float)
    void* stats;    // cat_fit scratch for (N, D, K, dt)
    size_t pca_bytes, lloyd_bytes, stats_bytes, bytes;
};
static PcaFitWs carve_pca_fit(void* base, int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt) {
    PcaFitWs w;
    w.pca_bytes = cat_pca_workspace_bytes(N, D, p, dt);
    const int32_t pp = pad4(p);
    w.lloyd_bytes = carve_fit(nullptr, N, pp, K, CAT_F32).bytes;
    w.stats_bytes = carve_fit(nullptr, N, D, K, dt).bytes;
    char* b = (char*)base;
    size_t off = 0;
    w.pca = b + off;
    off += align256(w.pca_bytes);
    w.z = (float*)(b + off);
    off += align256((size_t)N * (size_t)pp * sizeof(float));
    w.cz = (float*)(b + off);
    off += align256((size_t)K * (size_t)pp * sizeof(float));
    w.lloyd = b + off;
    off += align256(w.lloyd_bytes);
    w.stats = b + off;
    off += align256(w.stats_bytes);
    w.bytes = off;
    return w;
}

size_t cat_fit_pca_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt) || p < 1 || (int64_t)p > D || cat_pca_workspace_bytes(N, D, p, dt) == 0) return 0;
    return carve_pca_fit(nullptr, N, D, K, p, dt).bytes;
}

cat_status cat_fit_pca(const void* lq, const void* fp, int64_t N, int64_t D, int32_t K, int32_t p, int32_t iters, uint64_t seed,
                       cat_dtype dt, float* mean, float* components, float* centroids_z, float* gamma, float* beta,
                       int32_t* assignments, int32_t* counts, double* inertia, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
    CAT_TRY(check_shape("cat_fit_pca", N, D, K, dt));
    if (iters < 0) return set_error(CAT_ERR_INVALID_ARG, "cat_fit_pca: iters = %d is negative", (int)iters);
    if (p < 1 || (int64_t)p > D) return set_error(CAT_ERR_INVALID_ARG, "cat_fit_pca: need 1 <= p <= D (p=%d)", (int)p);
    CAT_TRY(check_ptr("cat_fit_pca", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "fp", fp, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "mean", mean, 4));
    CAT_TRY(check_ptr("cat_fit_pca", "components", components, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "centroids_z", centroids_z, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "gamma", gamma, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "beta", beta, 16));
    CAT_TRY(check_ptr("cat_fit_pca", "assignments", assignments, 4));
    if (cat_pca_workspace_bytes(N, D, p, dt) == 0)
        return set_error(CAT_ERR_UNSUPPORTED, "cat_fit_pca: the PCA front-end does not take D=%lld", (long long)D);
    PcaFitWs w = carve_pca_fit(workspace, N, D, K, p, dt);
    CAT_TRY(check_ws("cat_fit_pca", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    CAT_TRY(cat_pca_fit(lq, N, D, p, dt, 0, mean, components, nullptr, w.pca, w.pca_bytes, hip_stream));
    const int32_t pp = pad4(p);
    CAT_TRY(pca_project_ld(lq, N, D, p, dt, mean, components, w.z, pp, st));
    // clusters from the scores ...
    FitWs wz = carve_fit(w.lloyd, N, pp, K, CAT_F32);
    float* cz = pp == p ? centroids_z : w.cz;
    CAT_TRY(run_lloyd(w.z, CAT_F32, N, pp, K, iters, seed, nullptr, cz, assignments, inertia, wz, st));
    if (pp != p) CAT_TRY(launch_copy_cols(cz, K, pp, centroids_z, p, p, st));
    // ... the affine fit on the full vectors (rows are shared, so the counts and first rows carry over)
    FitWs wx = carve_fit(w.stats, N, D, K, dt);
    CAT_TRY(step_stats(lq, fp, dt, assignments, N, D, K, wz.counts, wz.rep, nullptr, wx, gamma, beta, st));
    if (counts) CAT_TRY(launch_copy_words(wz.counts, counts, K, st));
    return CAT_OK;
}

struct PcaApplyWs {
    float* z;    // N x pad4(p)
    float* cz;   // K x pad4(p)
    int32_t* assign;
    void* step;  // cat_fit scratch for (N, pad4(p), K, float): the assignment step
    size_t step_bytes, bytes;
};
static PcaApplyWs carve_pca_apply(void* base, int64_t N, int32_t K, int32_t p) {
    PcaApplyWs w;
    const int32_t pp = pad4(p);
    w.step_bytes = carve_fit(nullptr, N, pp, K, CAT_F32).bytes;
    char* b = (char*)base;
    size_t off = 0;
    w.z = (float*)(b + off);
    off += align256((size_t)N * (size_t)pp * sizeof(float));
    w.cz = (float*)(b + off);
    off += align256((size_t)K * (size_t)pp * sizeof(float));
    w.assign = (int32_t*)(b + off);
    off += align256((size_t)N * sizeof(int32_t));
    w.step = b + off;
    off += align256(w.step_bytes);
    w.bytes = off;
    return w;
}

size_t cat_apply_pca_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt) {
    if (!shape_ok(N, D, K, dt) || p < 1 || (int64_t)p > D) return 0;
    return carve_pca_apply(nullptr, N, K, p).bytes;
}

cat_status cat_apply_pca(const void* lq, int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt, const float* mean,
                         const float* components, const float* centroids_z, const float* gamma, const float* beta, float alpha,
                         void* corrected, int32_t* assignments, void* workspace, size_t workspace_bytes, void* hip_stream) {
    CAT_TRY(check_shape("cat_apply_pca", N, D, K, dt));
    if (p < 1 || (int64_t)p > D) return set_error(CAT_ERR_INVALID_ARG, "cat_apply_pca: need 1 <= p <= D (p=%d)", (int)p);
    CAT_TRY(check_ptr("cat_apply_pca", "lq", lq, 16));
    CAT_TRY(check_ptr("cat_apply_pca", "mean", mean, 4));
    CAT_TRY(check_ptr("cat_apply_pca", "components", components, 16));
    CAT_TRY(check_ptr("cat_apply_pca", "centroids_z", centroids_z, 16));
    CAT_TRY(check_ptr("cat_apply_pca", "gamma", gamma, 16));
    CAT_TRY(check_ptr("cat_apply_pca", "beta", beta, 16));
    CAT_TRY(check_ptr("cat_apply_pca", "corrected", corrected, 16));
    if (corrected == lq) return set_error(CAT_ERR_INVALID_ARG, "cat_apply_pca: corrected may not alias lq");
    if (!std::isfinite(alpha)) return set_error(CAT_ERR_INVALID_ARG, "cat_apply_pca: alpha is not finite");
    PcaApplyWs w = carve_pca_apply(workspace, N, K, p);
    CAT_TRY(check_ws("cat_apply_pca", workspace, workspace_bytes, w.bytes));
    hipStream_t st = (hipStream_t)hip_stream;
    // one kernel where the shape allows it (not with the streaming path forced: that selects the step-by-step sequence)
    if (g_path.load() != CAT_PATH_STREAM && apply_pca_fused_supported(lq, D, K, p, mean, components, gamma, beta, corrected))
        return launch_apply_pca_fused(lq, N, D, K, p, dt, mean, components, centroids_z, gamma, beta, alpha, corrected,
                                      assignments, st);
    int32_t* a = assignments ? assignments : w.assign;
    const int32_t pp = pad4(p);
    CAT_TRY(pca_project_ld(lq, N, D, p, dt, mean, components, w.z, pp, st));
    const float* cz = centroids_z;
    if (pp != p) {
        CAT_TRY(launch_copy_cols(centroids_z, K, p, w.cz, pp, p, st));
        cz = w.cz;
    }
    FitWs ws = carve_fit(w.step, N, pp, K, CAT_F32);
    CAT_TRY(step_assign(w.z, CAT_F32, N, pp, K, cz, a, nullptr, nullptr, nullptr, ws.tile, st));
    return cat_apply_assigned(lq, a, N, D, K, dt, gamma, beta, alpha, corrected, hip_stream);
}

}  // extern "C"
