// Host entry points of the C ABI declared in rls.h: argument checks, workspace carving, launches.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "rls_internal.h"

namespace rls {

static thread_local hipError_t g_last_hip = hipSuccess;
void set_hip_error(hipError_t e) { g_last_hip = e; }

// ---- benchmark timing: event pairs around the Lloyd step kernel --------------------------------
// (bench-only state, see rls_bench.h; everything below g_profile_mutex is guarded by it)
static std::atomic<bool> g_profile_on{false};
static std::mutex g_profile_mutex;
static std::vector<hipEvent_t> g_events;     // pool, reused
static size_t g_events_used = 0;             // events recorded since the last read (even: begin, odd: end)

bool profile_enabled() { return g_profile_on.load(std::memory_order_relaxed); }

hipError_t profile_mark(hipStream_t s, bool begin)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (begin != (g_events_used % 2 == 0)) return hipSuccess;   // keep pairs aligned
    if (g_events_used == g_events.size()) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) return e;
        g_events.push_back(ev);
    }
    return hipEventRecord(g_events[g_events_used++], s);
}

static int32_t check_matrix(const float *X, int64_t N, int32_t d, int64_t ldx)
{
    if (!X) return RLS_ERR_NULL;
    if (N < 1 || N > RLS_MAX_N || d < 1 || d > RLS_MAX_D) return RLS_ERR_INVALID_ARG;
    if (ldx < d) return RLS_ERR_SHAPE;
    return RLS_OK;
}

static int32_t check_forest(const rls_forest *f, int32_t d)
{
    if (!f) return RLS_ERR_NULL;
    if (!f->feat_dev || !f->thr_dev || !f->leaf_dev) return RLS_ERR_NULL;
    if (f->n_trees < 1 || f->depth < 1 || f->depth > RLS_MAX_DEPTH) return RLS_ERR_INVALID_ARG;
    if (f->n_features != d) return RLS_ERR_SHAPE;
    return RLS_OK;
}

static int32_t check_sweep(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t batch)
{
    if (N < 1 || N > RLS_MAX_N || d < 1 || d > RLS_MAX_D) return RLS_ERR_INVALID_ARG;
    if (k_min < 1 || k_max < k_min || k_max > RLS_MAX_K || (int64_t)k_max > N) return RLS_ERR_INVALID_ARG;
    if (batch < 1 || batch > RLS_MAX_BATCH) return RLS_ERR_INVALID_ARG;
    return RLS_OK;
}

}  // namespace rls

using namespace rls;

extern "C" {

int32_t rls_version(void) { return 133; }

const char *rls_error_string(int32_t code)
{
    switch (code) {
    case RLS_OK: return "ok";
    case RLS_ERR_INVALID_ARG: return "invalid argument (size, range or limit)";
    case RLS_ERR_NULL: return "required pointer is null";
    case RLS_ERR_SHAPE: return "shapes disagree";
    case RLS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RLS_ERR_HIP: return "HIP runtime error";
    case RLS_ERR_NOT_IMPLEMENTED: return "not implemented";
    default: return "unknown error code";
    }
}

int32_t rls_last_hip_error(void) { return (int32_t)g_last_hip; }

int32_t rls_profile_enable(int32_t on)
{
    g_profile_on.store(on != 0, std::memory_order_relaxed);
    return RLS_OK;
}

int32_t rls_profile_read(int32_t *n_launches, double *total_ms)
{
    if (!n_launches || !total_ms) return RLS_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    double sum = 0.0;
    const size_t pairs = g_events_used / 2;
    for (size_t i = 0; i < pairs; ++i) {
        RLS_HIP_TRY(hipEventSynchronize(g_events[2 * i + 1]));
        float ms = 0.0f;
        RLS_HIP_TRY(hipEventElapsedTime(&ms, g_events[2 * i], g_events[2 * i + 1]));
        sum += (double)ms;
    }
    g_events_used = 0;
    *n_launches = (int32_t)pairs;
    *total_ms = sum;
    return RLS_OK;
}

int32_t rls_gbt_score_batched(const rls_forest *forests, int32_t batch, const float *X_dev, int64_t N, int32_t d,
                              int64_t ldx, int64_t x_batch_stride, float *score_dev, void *stream)
{
    if (!forests || !score_dev) return RLS_ERR_NULL;
    if (batch < 1 || batch > RLS_MAX_BATCH) return RLS_ERR_INVALID_ARG;
    int32_t rc = check_matrix(X_dev, N, d, ldx);
    if (rc != RLS_OK) return rc;
    if (batch > 1 && x_batch_stride < N * ldx - (ldx - d)) return RLS_ERR_SHAPE;
    std::vector<ForestArgs> fa((size_t)batch);
    for (int32_t b = 0; b < batch; ++b) {
        rc = check_forest(&forests[b], d);
        if (rc != RLS_OK) return rc;
        fa[b] = ForestArgs{forests[b].n_trees, forests[b].depth, forests[b].base, forests[b].feat_dev,
                           forests[b].thr_dev, forests[b].leaf_dev};
    }
    RLS_HIP_TRY(launch_gbt_score(fa.data(), batch, X_dev, N, d, ldx, x_batch_stride, score_dev, (hipStream_t)stream));
    return RLS_OK;
}

int32_t rls_gbt_score(const rls_forest *forest, const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                      float *score_dev, void *stream)
{
    return rls_gbt_score_batched(forest, 1, X_dev, N, d, ldx, 0, score_dev, stream);
}

int64_t rls_kmeans_sweep_workspace_bytes(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t batch)
{
    const int32_t rc = check_sweep(N, d, k_min, k_max, batch);
    if (rc != RLS_OK) return rc;
    SweepPlan plan;
    const int32_t prc = make_sweep_plan(N, d, k_min, k_max, batch, &plan);
    if (prc != RLS_OK) return prc;
    SweepLayout L;
    sweep_layout(plan, N, d, k_max, batch, &L);
    return L.total;
}

int32_t rls_kmeanspp_chain(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_max, uint64_t seed,
                           int64_t *init_idx_dev, void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    int32_t rc = check_matrix(X_dev, N, d, ldx);
    if (rc != RLS_OK) return rc;
    if (!init_idx_dev) return RLS_ERR_NULL;
    rc = check_sweep(N, d, k_max, k_max, 1);
    if (rc != RLS_OK) return rc;
    SweepPlan plan;
    rc = make_sweep_plan(N, d, k_max, k_max, 1, &plan);
    if (rc != RLS_OK) return rc;
    SweepLayout L;
    sweep_layout(plan, N, d, k_max, 1, &L);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < L.total) return RLS_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace_dev);
    RLS_HIP_TRY(launch_seed_chain(X_dev, N, d, ldx, 0, 1, k_max, &seed, init_idx_dev, k_max, ws, L, (hipStream_t)stream));
    return RLS_OK;
}

int32_t rls_kmeans_sweep_batched(int32_t batch, const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                                 int64_t x_batch_stride, int32_t k_min, int32_t k_max, int32_t iters,
                                 const uint64_t *seeds, const int64_t *init_idx_dev, int32_t *labels_dev,
                                 float *centroids_dev, double *inertia_dev, double *inertia_trace_dev,
                                 int32_t *status_dev, void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    int32_t rc = check_matrix(X_dev, N, d, ldx);
    if (rc != RLS_OK) return rc;
    rc = check_sweep(N, d, k_min, k_max, batch);
    if (rc != RLS_OK) return rc;
    if (!centroids_dev || !inertia_dev || !status_dev) return RLS_ERR_NULL;
    if (!init_idx_dev && !seeds) return RLS_ERR_NULL;
    if (iters < 0) return RLS_ERR_INVALID_ARG;
    if (ldx > RLS_MAX_LDX) return RLS_ERR_SHAPE;   // the step kernel addresses a slab of rows with 32-bit offsets
    if (batch > 1 && x_batch_stride < N * ldx - (ldx - d)) return RLS_ERR_SHAPE;
    SweepPlan plan;
    rc = make_sweep_plan(N, d, k_min, k_max, batch, &plan);
    if (rc != RLS_OK) return rc;
    SweepLayout L;
    sweep_layout(plan, N, d, k_max, batch, &L);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < L.total) return RLS_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace_dev);
    hipStream_t s = (hipStream_t)stream;

    const int64_t *init = init_idx_dev;
    int64_t init_bs = k_max;
    if (!init) {
        int64_t *chain = reinterpret_cast<int64_t *>(ws + L.chain);
        RLS_HIP_TRY(launch_seed_chain(X_dev, N, d, ldx, x_batch_stride, batch, k_max, seeds, chain, L.per_batch / 8, ws, L, s));
        init = chain;
        init_bs = L.per_batch / 8;
    }
    SweepArgs a;
    a.X = X_dev; a.N = N; a.d = d; a.ldx = ldx; a.x_batch_stride = x_batch_stride; a.batch = batch; a.iters = iters;
    a.init_idx = init; a.init_batch_stride = init_bs;
    a.labels = labels_dev; a.centroids = centroids_dev; a.inertia = inertia_dev; a.trace = inertia_trace_dev;
    a.status = status_dev; a.ws = ws;
    a.reuse_colstats = 0; a.reuse_prepared = 0;
    RLS_HIP_TRY(launch_sweep(plan, L, a, s));
    return RLS_OK;
}

int32_t rls_kmeans_sweep(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_min, int32_t k_max,
                         int32_t iters, uint64_t seed, const int64_t *init_idx_dev, int32_t *labels_dev,
                         float *centroids_dev, double *inertia_dev, double *inertia_trace_dev, int32_t *status_dev,
                         void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    return rls_kmeans_sweep_batched(1, X_dev, N, d, ldx, 0, k_min, k_max, iters, &seed, init_idx_dev, labels_dev,
                                    centroids_dev, inertia_dev, inertia_trace_dev, status_dev, workspace_dev,
                                    workspace_bytes, stream);
}

static int32_t until_knee_workspace(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t k_wave, int64_t *bytes)
{
    int64_t need = 0;
    for (int32_t k_lo = k_min; k_lo <= k_max; k_lo += k_wave) {
        const int32_t k_hi = k_lo + k_wave - 1 < k_max ? k_lo + k_wave - 1 : k_max;
        SweepPlan plan;
        const int32_t rc = make_sweep_plan(N, d, k_lo, k_hi, 1, &plan);
        if (rc != RLS_OK) return rc;
        SweepLayout L;
        sweep_layout(plan, N, d, k_max, 1, &L);     // chain sized for k_max: the leading blocks sit at the same offsets in every wave
        if (L.total > need) need = L.total;
    }
    *bytes = need;
    return RLS_OK;
}

int64_t rls_kmeans_sweep_until_knee_workspace_bytes(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t k_wave)
{
    const int32_t rc = check_sweep(N, d, k_min, k_max, 1);
    if (rc != RLS_OK) return rc;
    if (k_wave < 1) return RLS_ERR_INVALID_ARG;
    int64_t bytes = 0;
    const int32_t wrc = until_knee_workspace(N, d, k_min, k_max, k_wave, &bytes);
    return wrc != RLS_OK ? wrc : bytes;
}

int32_t rls_kmeans_sweep_until_knee(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_min, int32_t k_max,
                                    int32_t k_wave, int32_t iters, uint64_t seed, const int64_t *init_idx_dev,
                                    double knee_const, int32_t *labels_dev, float *centroids_dev, double *inertia_dev,
                                    double *inertia_host, int32_t *k_out, int32_t *n_done_out, int32_t *status_dev,
                                    void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    int32_t rc = check_matrix(X_dev, N, d, ldx);
    if (rc != RLS_OK) return rc;
    rc = check_sweep(N, d, k_min, k_max, 1);
    if (rc != RLS_OK) return rc;
    if (!centroids_dev || !inertia_dev || !inertia_host || !k_out || !n_done_out || !status_dev) return RLS_ERR_NULL;
    if (iters < 0 || k_wave < 1) return RLS_ERR_INVALID_ARG;
    if (ldx > RLS_MAX_LDX) return RLS_ERR_SHAPE;
    int64_t need = 0;
    rc = until_knee_workspace(N, d, k_min, k_max, k_wave, &need);
    if (rc != RLS_OK) return rc;
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < need) return RLS_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace_dev);
    hipStream_t s = (hipStream_t)stream;

    double previous_loss = INFINITY;
    int32_t chosen = k_max, n_done = 0, chain_done = 0;
    bool fired = false, have_colstats = false, have_prepared = false;
    for (int32_t k_lo = k_min; k_lo <= k_max && !fired; k_lo += k_wave) {
        const int32_t k_hi = k_lo + k_wave - 1 < k_max ? k_lo + k_wave - 1 : k_max;
        SweepPlan plan;
        rc = make_sweep_plan(N, d, k_lo, k_hi, 1, &plan);
        if (rc != RLS_OK) return rc;
        SweepLayout L;
        sweep_layout(plan, N, d, k_max, 1, &L);
        const int64_t *init = init_idx_dev;
        if (!init) {
            // the chain grows with the waves: centres chain_done .. k_hi-1 are drawn now, from the distance state of the earlier ones
            int64_t *chain = reinterpret_cast<int64_t *>(ws + L.chain);
            RLS_HIP_TRY(launch_seed_chain(X_dev, N, d, ldx, 0, 1, k_hi, &seed, chain, k_max, ws, L, s, chain_done));
            chain_done = k_hi;
            init = chain;
        }
        const int64_t row0 = rows_before(k_min, k_lo - k_min);
        SweepArgs a;
        a.X = X_dev; a.N = N; a.d = d; a.ldx = ldx; a.x_batch_stride = 0; a.batch = 1; a.iters = iters;
        a.init_idx = init; a.init_batch_stride = k_max;
        a.labels = labels_dev ? labels_dev + (int64_t)(k_lo - k_min) * N : nullptr;
        a.centroids = centroids_dev + row0 * d;
        a.inertia = inertia_dev + (k_lo - k_min);
        a.trace = nullptr;
        a.status = status_dev; a.ws = ws;
        // every wave sweeps the same rows with the same workspace: column information and prepared copy are made once
        a.reuse_colstats = have_colstats ? 1 : 0;
        a.reuse_prepared = have_prepared ? 1 : 0;
        RLS_HIP_TRY(launch_sweep(plan, L, a, s));
        have_colstats = true;
        if (sweep_uses_prepared(plan, iters, false)) have_prepared = true;
        int32_t status_host = 0;
        RLS_HIP_TRY(hipMemcpyAsync(inertia_host + (k_lo - k_min), inertia_dev + (k_lo - k_min),
                                   (size_t)(k_hi - k_lo + 1) * sizeof(double), hipMemcpyDeviceToHost, s));
        RLS_HIP_TRY(hipMemcpyAsync(&status_host, status_dev, sizeof(int32_t), hipMemcpyDeviceToHost, s));
        RLS_HIP_TRY(hipStreamSynchronize(s));
        n_done = k_hi - k_min + 1;
        if (status_host != 0) { chosen = 0; break; }      // the data broke a precondition: see status_dev
        for (int32_t k = k_lo; k <= k_hi; ++k) {
            const double loss = inertia_host[k - k_min];
            if (knee_const * loss > previous_loss) { chosen = k; fired = true; break; }
            previous_loss = loss;
        }
    }
    *k_out = chosen;
    *n_done_out = n_done;
    return RLS_OK;
}

int32_t rls_pick_knee(const double *inertia_host, int32_t k_min, int32_t k_max, double knee_const, int32_t *k_out)
{
    if (!inertia_host || !k_out) return RLS_ERR_NULL;
    if (k_min < 1 || k_max < k_min) return RLS_ERR_INVALID_ARG;
    double previous_loss = INFINITY;
    int32_t chosen = k_max;
    for (int32_t k = k_min; k <= k_max; ++k) {
        const double loss = inertia_host[k - k_min];
        if (knee_const * loss > previous_loss) { chosen = k; break; }
        previous_loss = loss;
    }
    *k_out = chosen;
    return RLS_OK;
}

int32_t rls_snap_to_valid_batched(int32_t batch, const float *centroids_dev, int32_t k, int32_t d, int64_t ldc,
                                  int64_t c_batch_stride, const rls_knob_domains *domains, int32_t *cfg_dev, void *stream)
{
    if (!centroids_dev || !domains || !cfg_dev) return RLS_ERR_NULL;
    if (batch < 1 || batch > RLS_MAX_BATCH || k < 1 || d < 1 || d > RLS_MAX_D) return RLS_ERR_INVALID_ARG;
    if (ldc < d) return RLS_ERR_SHAPE;
    std::vector<DomainArgs> da((size_t)batch);
    for (int32_t b = 0; b < batch; ++b) {
        if (!domains[b].offsets_dev || !domains[b].values_dev) return RLS_ERR_NULL;
        if (domains[b].n_knobs < 1 || domains[b].n_knobs > d) return RLS_ERR_SHAPE;
        if (domains[b].n_knobs != domains[0].n_knobs) return RLS_ERR_SHAPE;
        da[b] = DomainArgs{domains[b].n_knobs, domains[b].offsets_dev, domains[b].values_dev};
    }
    RLS_HIP_TRY(launch_snap(da.data(), batch, centroids_dev, k, d, ldc, c_batch_stride, cfg_dev, (hipStream_t)stream));
    return RLS_OK;
}

int32_t rls_snap_to_valid(const float *centroids_dev, int32_t k, int32_t d, int64_t ldc,
                          const rls_knob_domains *domains, int32_t *cfg_dev, void *stream)
{
    return rls_snap_to_valid_batched(1, centroids_dev, k, d, ldc, 0, domains, cfg_dev, stream);
}

int32_t rls_knob_modes(const float *X_dev, int64_t N, int32_t d, int64_t ldx, const rls_knob_domains *domains,
                       int32_t n_total_values, int32_t *mode_cfg_dev, int32_t *hist_dev, void *stream)
{
    const int32_t rc = check_matrix(X_dev, N, d, ldx);
    if (rc != RLS_OK) return rc;
    if (!domains || !mode_cfg_dev || !hist_dev) return RLS_ERR_NULL;
    if (!domains->offsets_dev || !domains->values_dev) return RLS_ERR_NULL;
    if (domains->n_knobs < 1 || domains->n_knobs > d) return RLS_ERR_SHAPE;
    if (n_total_values < domains->n_knobs || n_total_values > RLS_MAX_DOMAIN_VALUES) return RLS_ERR_INVALID_ARG;
    const DomainArgs dm{domains->n_knobs, domains->offsets_dev, domains->values_dev};
    RLS_HIP_TRY(launch_knob_modes(X_dev, N, ldx, dm, n_total_values, mode_cfg_dev, hist_dev, (hipStream_t)stream));
    return RLS_OK;
}

int32_t rls_replace_visited(int32_t *cfg_dev, int32_t k, int32_t n_knobs, const int32_t *visited_dev,
                            int64_t n_visited, const int32_t *mode_cfg_dev, int32_t *replaced_dev, void *stream)
{
    if (!cfg_dev || !mode_cfg_dev || !replaced_dev) return RLS_ERR_NULL;
    if (k < 1 || k > 65535 || n_knobs < 1 || n_knobs > RLS_MAX_D || n_visited < 0) return RLS_ERR_INVALID_ARG;
    if (n_visited > 0 && !visited_dev) return RLS_ERR_NULL;
    RLS_HIP_TRY(launch_replace_visited(cfg_dev, k, n_knobs, visited_dev, n_visited, mode_cfg_dev, replaced_dev,
                                       (hipStream_t)stream));
    return RLS_OK;
}

int32_t rls_apply_actions(const int32_t *cfg_dev, const int8_t *action_dev, int64_t m, const rls_knob_domains *domains,
                          int32_t *cfg_out_dev, float *features_dev, int64_t ldf, void *stream)
{
    if (!cfg_dev || !action_dev || !domains || !cfg_out_dev) return RLS_ERR_NULL;
    if (!domains->offsets_dev || !domains->values_dev) return RLS_ERR_NULL;
    if (m < 1 || m > ((int64_t)1 << 31) || domains->n_knobs < 1 || domains->n_knobs > RLS_MAX_D) return RLS_ERR_INVALID_ARG;
    if (features_dev && ldf < domains->n_knobs) return RLS_ERR_SHAPE;
    const DomainArgs dm{domains->n_knobs, domains->offsets_dev, domains->values_dev};
    RLS_HIP_TRY(launch_apply_actions(cfg_dev, reinterpret_cast<const signed char *>(action_dev), m, dm, cfg_out_dev,
                                     features_dev, ldf, (hipStream_t)stream));
    return RLS_OK;
}

}  // extern "C"
