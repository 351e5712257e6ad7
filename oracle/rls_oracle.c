/*
 * CPU oracle for the adaptive-sampling hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, sequential statement of what the path computes, written from
 * the paper: the cost-model query of Sec. 4.1 ("Reward formulation" and
 * "Learning procedure": every configuration of a trajectory is scored by the
 * boosted-tree model) and Algorithm 1 of Sec. 4.2 (k-means for a range of k,
 * the knee test on the loss curve, centroids handed on as the next samples).
 * Nothing here is shared with the GPU library, and nothing outside the tests,
 * the smoke check and the benchmark's CPU-baseline leg may call it.
 *
 * Arithmetic: inputs are fp32; distances, losses and comparisons are fp64 in
 * the direct form sum_l (x_l - c_l)^2, summed over l in ascending order with a
 * separately rounded multiply and add; a centroid is the mean of its members
 * computed from the EXACT sum (128-bit fixed point, so the order of summation
 * does not matter), rounded once to fp64, divided by the count in fp64 and
 * rounded to fp32.
 *
 * Pins (tests/test_oracle_*.py): tree scoring against a NumPy re-walk, stumps
 * and +-inf thresholds; the seeding draw against its D^2 law, SplitMix64 test
 * vectors and the prefix property; Lloyd against brute force over all
 * labelings, monotone loss over every half step, planted clusters, closed
 * forms for k = 1 and k = N, exact means via rationals; the draw's boundary
 * branch and the two-nearest helper of the parity tests against NumPy brute
 * force; the knee rule against
 * hand-made curves following Algorithm 1; snapping against brute force.
 * The whole chain has no numeric example in the paper: parity unpinned against
 * the paper beyond those properties.
 *
 * Only the loop over points in the assignment step carries an OpenMP pragma.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_RANGE (-2) /* a value cannot be held exactly in the fixed-point sum */
#define ORC_ERR_NOMEM (-3)

/* ------------------------------------------------------------------------ */
/* Cost-model query (Sec. 4.1): sum of leaf values of complete binary trees. */
/* Node n of a tree has children 2n+1 (taken when x[feat] < thr) and 2n+2.   */
/* score32 adds the leaves in tree order in fp32, score64 in fp64.           */
int32_t orc_gbt_score(int32_t n_trees, int32_t depth, int32_t n_features, float base,
                      const int32_t *feat, const float *thr, const float *leaf,
                      const float *X, int64_t N, int32_t d, int64_t ldx,
                      float *score32, double *score64)
{
    if (!feat || !thr || !leaf || !X || !score32) return ORC_ERR_ARG;
    if (n_trees < 1 || depth < 1 || depth > 12 || n_features != d || N < 0 || ldx < d) return ORC_ERR_ARG;
    const int64_t n_int = ((int64_t)1 << depth) - 1, n_leaf = (int64_t)1 << depth;
    for (int64_t i = 0; i < N; ++i) {
        const float *x = X + i * ldx;
        float s32 = base;
        double s64 = (double)base;
        for (int32_t t = 0; t < n_trees; ++t) {
            int64_t n = 0;
            for (int32_t lev = 0; lev < depth; ++lev) {
                const int32_t f = feat[t * n_int + n];
                if (f < 0 || f >= d) return ORC_ERR_ARG;
                n = 2 * n + 1 + (x[f] < thr[t * n_int + n] ? 0 : 1);
            }
            const float v = leaf[t * n_leaf + (n - n_int)];
            s32 = s32 + v;
            s64 = s64 + (double)v;
        }
        score32[i] = s32;
        if (score64) score64[i] = s64;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Counter-based uniform draws: SplitMix64 (Steele, Lea, Flood 2014) applied */
/* to seed + (j+1)*golden-gamma; the top 53 bits give a double in [0,1).     */
uint64_t orc_splitmix64(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

double orc_uniform(uint64_t seed, uint64_t j)
{
    return (double)(orc_splitmix64(seed, j) >> 11) * 0x1.0p-53;
}

static double sqdist(const float *x, const float *c, int32_t d)
{
    double acc = 0.0;
    for (int32_t l = 0; l < d; ++l) {
        const double diff = (double)x[l] - (double)c[l];
        const double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

/* ------------------------------------------------------------------------ */
/* The D^2 draw: the first index whose inclusive prefix sum of D (taken in   */
/* index order) exceeds r.  When no prefix does - r was rounded up to the    */
/* total - the last index with D > 0 is taken; -1 when no D is positive.     */
int64_t orc_draw_index(const double *D, int64_t N, double r)
{
    double prefix = 0.0;
    int64_t last_pos = -1;
    for (int64_t i = 0; i < N; ++i) {
        prefix = prefix + D[i];
        if (D[i] > 0.0) last_pos = i;
        if (prefix > r) return i;
    }
    return last_pos;
}

/* ------------------------------------------------------------------------ */
/* Seeding: one k-means++ chain (D^2 sampling) of k_max centres.  A run with */
/* k clusters starts from the first k of them.  The paper does not say how   */
/* k-means is initialised; the workload definition asks for k-means++.       */
int32_t orc_kmeanspp_chain(const float *X, int64_t N, int32_t d, int64_t ldx,
                           int32_t k_max, uint64_t seed, int64_t *idx_out)
{
    if (!X || !idx_out || N < 1 || d < 1 || ldx < d || k_max < 1 || k_max > N) return ORC_ERR_ARG;
    double *D = (double *)malloc(sizeof(double) * (size_t)N);
    if (!D) return ORC_ERR_NOMEM;
    int64_t first = (int64_t)(orc_uniform(seed, 0) * (double)N);
    if (first >= N) first = N - 1;
    idx_out[0] = first;
    for (int32_t j = 1; j < k_max; ++j) {
        const float *c = X + idx_out[j - 1] * ldx;
        double S = 0.0;
        for (int64_t i = 0; i < N; ++i) {
            const double dist = sqdist(X + i * ldx, c, d);
            if (j == 1 || dist < D[i]) D[i] = dist;
            S = S + D[i];
        }
        int64_t pick = -1;
        if (S > 0.0) {
            pick = orc_draw_index(D, N, orc_uniform(seed, (uint64_t)j) * S);
        } else {
            /* every point coincides with a chosen centre: smallest index not chosen yet */
            for (int64_t i = 0; i < N && pick < 0; ++i) {
                int taken = 0;
                for (int32_t m = 0; m < j; ++m) taken |= (idx_out[m] == i);
                if (!taken) pick = i;
            }
        }
        idx_out[j] = pick;
    }
    free(D);
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Exact column sums: every fp32 value that is a multiple of 2^-60 and below */
/* 2^40 in magnitude becomes an integer after scaling by 2^60; up to 2^26 of */
/* them add without overflow in 128 bits.                                    */
#define FIX_SHIFT 0x1.0p60
#define FIX_UNSHIFT 0x1.0p-60

static int to_fixed(float x, __int128 *q)
{
    const double s = (double)x * FIX_SHIFT;
    if (!(fabs(s) < 0x1.0p100) || s != floor(s)) return 0;
    *q = (__int128)s;
    return 1;
}

/* assignment of every point to its nearest centroid; ties go to the lowest index */
static double assign_all(const float *X, int64_t N, int32_t d, int64_t ldx,
                         const float *C, int32_t k, int32_t *label, double *mind)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double best = INFINITY;
        int32_t arg = 0;
        for (int32_t j = 0; j < k; ++j) {
            const double dist = sqdist(X + i * ldx, C + (int64_t)j * d, d);
            if (dist < best) { best = dist; arg = j; }
        }
        label[i] = arg;
        mind[i] = best;
    }
    double J = 0.0;
    for (int64_t i = 0; i < N; ++i) J = J + mind[i];
    return J;
}

/* loss of a given labelling against given centroids */
static double loss_of(const float *X, int64_t N, int32_t d, int64_t ldx,
                      const float *C, const int32_t *label)
{
    double J = 0.0;
    for (int64_t i = 0; i < N; ++i) J = J + sqdist(X + i * ldx, C + (int64_t)label[i] * d, d);
    return J;
}

/*
 * Lloyd iteration for one k with a fixed number of rounds (no early stop):
 *   C^0 = X[init_idx[0..k-1]];  for t < iters: l^t = assign(C^t); C^{t+1} = means(l^t)
 * (a centroid that lost all its points keeps its previous value);
 * finally l = assign(C^iters) and the loss is measured against C^iters.
 * half_trace, if given, receives 2*iters+1 values:
 *   J(l^0,C^0), J(l^0,C^1), J(l^1,C^1), ..., J(l^iters, C^iters).
 */
int32_t orc_lloyd(const float *X, int64_t N, int32_t d, int64_t ldx, int32_t k, int32_t iters,
                  const int64_t *init_idx, int32_t *labels, float *centroids,
                  double *inertia, double *half_trace)
{
    if (!X || !init_idx || !labels || !centroids || !inertia) return ORC_ERR_ARG;
    if (N < 1 || d < 1 || ldx < d || k < 1 || k > N || iters < 0 || N > ((int64_t)1 << 26)) return ORC_ERR_ARG;
    for (int32_t j = 0; j < k; ++j) {
        if (init_idx[j] < 0 || init_idx[j] >= N) return ORC_ERR_ARG;
        memcpy(centroids + (int64_t)j * d, X + init_idx[j] * ldx, sizeof(float) * (size_t)d);
    }
    double *mind = (double *)malloc(sizeof(double) * (size_t)N);
    __int128 *sum = (__int128 *)malloc(sizeof(__int128) * (size_t)k * (size_t)d);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
    if (!mind || !sum || !cnt) { free(mind); free(sum); free(cnt); return ORC_ERR_NOMEM; }
    int32_t rc = ORC_OK;
    for (int32_t t = 0; t < iters && rc == ORC_OK; ++t) {
        const double J = assign_all(X, N, d, ldx, centroids, k, labels, mind);
        if (half_trace) half_trace[2 * t] = J;
        memset(sum, 0, sizeof(__int128) * (size_t)k * (size_t)d);
        memset(cnt, 0, sizeof(int64_t) * (size_t)k);
        for (int64_t i = 0; i < N && rc == ORC_OK; ++i) {
            const int32_t j = labels[i];
            cnt[j] += 1;
            for (int32_t l = 0; l < d; ++l) {
                __int128 q;
                if (!to_fixed(X[i * ldx + l], &q)) { rc = ORC_ERR_RANGE; break; }
                sum[(int64_t)j * d + l] += q;
            }
        }
        if (rc != ORC_OK) break;
        for (int32_t j = 0; j < k; ++j) {
            if (cnt[j] == 0) continue;
            for (int32_t l = 0; l < d; ++l) {
                const double total = (double)sum[(int64_t)j * d + l] * FIX_UNSHIFT;
                centroids[(int64_t)j * d + l] = (float)(total / (double)cnt[j]);
            }
        }
        if (half_trace) half_trace[2 * t + 1] = loss_of(X, N, d, ldx, centroids, labels);
    }
    if (rc == ORC_OK) {
        *inertia = assign_all(X, N, d, ldx, centroids, k, labels, mind);
        if (half_trace) half_trace[2 * iters] = *inertia;
    }
    free(mind); free(sum); free(cnt);
    return rc;
}

/*
 * The loop over k of Algorithm 1 without the early break: every k in
 * [k_min, k_max] is clustered independently from the same seeding chain.
 * centroids are packed run after run (run k starts at d * sum_{k_min<=k'<k} k');
 * labels (optional) is [n_k][N]; inertia is [n_k];
 * trace (optional) is [n_k][iters+1] = J(l^t, C^t), t = 0..iters.
 */
int32_t orc_kmeans_sweep(const float *X, int64_t N, int32_t d, int64_t ldx,
                         int32_t k_min, int32_t k_max, int32_t iters, uint64_t seed,
                         const int64_t *init_idx, int32_t *labels, float *centroids,
                         double *inertia, double *trace)
{
    if (!X || !centroids || !inertia || k_min < 1 || k_max < k_min || k_max > N) return ORC_ERR_ARG;
    int64_t *chain = (int64_t *)malloc(sizeof(int64_t) * (size_t)k_max);
    int32_t *lab = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    double *half = (double *)malloc(sizeof(double) * (size_t)(2 * iters + 1));
    if (!chain || !lab || !half) { free(chain); free(lab); free(half); return ORC_ERR_NOMEM; }
    int32_t rc = ORC_OK;
    if (init_idx) memcpy(chain, init_idx, sizeof(int64_t) * (size_t)k_max);
    else rc = orc_kmeanspp_chain(X, N, d, ldx, k_max, seed, chain);
    int64_t off = 0;
    for (int32_t k = k_min; k <= k_max && rc == ORC_OK; ++k) {
        const int32_t r = k - k_min;
        int32_t *out_lab = labels ? labels + (int64_t)r * N : lab;
        rc = orc_lloyd(X, N, d, ldx, k, iters, chain, out_lab, centroids + off, inertia + r, half);
        if (trace && rc == ORC_OK)
            for (int32_t t = 0; t <= iters; ++t) trace[(int64_t)r * (iters + 1) + t] = half[2 * t];
        off += (int64_t)k * d;
    }
    free(chain); free(lab); free(half);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Knee test of Algorithm 1: walk k upward with PreviousLoss = infinity and  */
/* stop at the first k with Constant * Loss_k > PreviousLoss.  The centroids */
/* of that k were assigned before the test, so that k is the one kept; when  */
/* the test never fires the last k is kept.                                  */
int32_t orc_pick_knee(const double *inertia, int32_t k_min, int32_t k_max, double knee_const, int32_t *k_out)
{
    if (!inertia || !k_out || k_min < 1 || k_max < k_min) return ORC_ERR_ARG;
    double previous = INFINITY;
    for (int32_t k = k_min; k <= k_max; ++k) {
        const double loss = inertia[k - k_min];
        if (knee_const * loss > previous) { *k_out = k; return ORC_OK; }
        previous = loss;
    }
    *k_out = k_max;
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* NextSamples = Centroids (Algorithm 1): a centroid becomes a configuration */
/* by taking, knob by knob, the nearest value of that knob's domain (the     */
/* design space is the product of the knob domains, Sec. 2.2); ties go to    */
/* the lower index.  Knob j reads feature column j.                          */
int32_t orc_snap_to_valid(const float *centroids, int32_t k, int32_t d, int64_t ldc,
                          int32_t n_knobs, const int32_t *offsets, const float *values, int32_t *cfg)
{
    if (!centroids || !offsets || !values || !cfg || k < 1 || n_knobs < 1 || n_knobs > d || ldc < d) return ORC_ERR_ARG;
    for (int32_t j = 0; j < n_knobs; ++j)
        if (offsets[j + 1] <= offsets[j]) return ORC_ERR_ARG;
    for (int32_t i = 0; i < k; ++i) {
        for (int32_t j = 0; j < n_knobs; ++j) {
            const double c = (double)centroids[i * ldc + j];
            double best = INFINITY;
            int32_t arg = 0;
            for (int32_t v = offsets[j]; v < offsets[j + 1]; ++v) {
                const double gap = fabs(c - (double)values[v]);
                if (gap < best) { best = gap; arg = v - offsets[j]; }
            }
            cfg[i * n_knobs + j] = arg;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* mode(s_Theta) of Algorithm 1, read as Sec. 4.2 states it: the             */
/* configuration made of the mode of each dimension.  A point's value in      */
/* knob j is the domain entry nearest to its coordinate j (as in the snap    */
/* above); the mode is the entry most points take, the lowest index among    */
/* equally frequent ones.  hist (optional) receives the counts of all        */
/* entries, laid out like values.                                             */
int32_t orc_knob_modes(const float *X, int64_t N, int32_t d, int64_t ldx, int32_t n_knobs, const int32_t *offsets,
                       const float *values, int32_t *mode_cfg, int64_t *hist)
{
    if (!X || !offsets || !values || !mode_cfg || N < 1 || n_knobs < 1 || n_knobs > d || ldx < d) return ORC_ERR_ARG;
    for (int32_t j = 0; j < n_knobs; ++j)
        if (offsets[j + 1] <= offsets[j]) return ORC_ERR_ARG;
    int64_t *count = (int64_t *)calloc((size_t)offsets[n_knobs], sizeof(int64_t));
    if (!count) return ORC_ERR_ARG;
    for (int64_t i = 0; i < N; ++i) {
        for (int32_t j = 0; j < n_knobs; ++j) {
            const double x = (double)X[i * ldx + j];
            double best = INFINITY;
            int32_t arg = offsets[j];
            for (int32_t v = offsets[j]; v < offsets[j + 1]; ++v) {
                const double gap = fabs(x - (double)values[v]);
                if (gap < best) { best = gap; arg = v; }
            }
            count[arg] += 1;
        }
    }
    for (int32_t j = 0; j < n_knobs; ++j) {
        int32_t arg = offsets[j];
        for (int32_t v = offsets[j] + 1; v < offsets[j + 1]; ++v)
            if (count[v] > count[arg]) arg = v;
        mode_cfg[j] = arg - offsets[j];
    }
    if (hist) memcpy(hist, count, (size_t)offsets[n_knobs] * sizeof(int64_t));
    free(count);
    return ORC_OK;
}

/* The last loop of Algorithm 1: a sample that is already among the visited  */
/* configurations v_Theta is replaced by mode(s_Theta).  Configurations are  */
/* rows of n_knobs domain indices; replaced[i] tells which rows changed.      */
int32_t orc_replace_visited(int32_t *cfg, int32_t k, int32_t n_knobs, const int32_t *visited, int64_t n_visited,
                            const int32_t *mode_cfg, int32_t *replaced)
{
    if (!cfg || !mode_cfg || !replaced || k < 1 || n_knobs < 1 || n_visited < 0 || (n_visited > 0 && !visited)) return ORC_ERR_ARG;
    for (int32_t i = 0; i < k; ++i) {
        int32_t found = 0;
        for (int64_t v = 0; v < n_visited && !found; ++v) {
            int32_t same = 1;
            for (int32_t j = 0; j < n_knobs; ++j)
                if (visited[v * n_knobs + j] != cfg[i * n_knobs + j]) { same = 0; break; }
            found = same;
        }
        replaced[i] = found;
        if (found)
            for (int32_t j = 0; j < n_knobs; ++j) cfg[i * n_knobs + j] = mode_cfg[j];
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------ */
/* Configuration updater of the search agent (Sec. 4.1, "Action space" and    */
/* "Learning procedure"): an action is one direction per dimension -         */
/* decrement, stay or increment - and applying it to a configuration gives   */
/* the next one.  Configurations are rows of domain indices; a step that     */
/* would leave a knob's domain stays at its border (the paper is silent on   */
/* the border).  features (optional, [m][ldf]) receives the domain values of */
/* the new configurations in its first n_knobs columns, the form in which    */
/* the cost model is queried.                                                 */
int32_t orc_apply_actions(const int32_t *cfg, const int8_t *action, int64_t m, int32_t n_knobs, const int32_t *offsets,
                          const float *values, int32_t *cfg_out, float *features, int64_t ldf)
{
    if (!cfg || !action || !offsets || !cfg_out || m < 1 || n_knobs < 1) return ORC_ERR_ARG;
    if (features && (!values || ldf < n_knobs)) return ORC_ERR_ARG;
    for (int64_t i = 0; i < m; ++i) {
        for (int32_t j = 0; j < n_knobs; ++j) {
            const int32_t size = offsets[j + 1] - offsets[j];
            const int32_t a = action[i * n_knobs + j];
            if (size < 1 || a < -1 || a > 1) return ORC_ERR_ARG;
            int32_t v = cfg[i * n_knobs + j];
            if (v < 0 || v >= size) return ORC_ERR_ARG;
            v += a;
            if (v < 0) v = 0;
            if (v > size - 1) v = size - 1;
            cfg_out[i * n_knobs + j] = v;
            if (features) features[i * ldf + j] = values[offsets[j] + v];
        }
    }
    return ORC_OK;
}

/* threads the annotated assignment loop runs on */
int32_t orc_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* two smallest direct-form distances of one point (for the near-tie rule of the parity tests) */
int32_t orc_two_nearest(const float *x, int32_t d, const float *C, int32_t k, double *d1, double *d2, int32_t *arg)
{
    if (!x || !C || !d1 || !d2 || !arg || k < 1) return ORC_ERR_ARG;
    double a = INFINITY, b = INFINITY;
    int32_t ia = 0;
    for (int32_t j = 0; j < k; ++j) {
        const double dist = sqdist(x, C + (int64_t)j * d, d);
        if (dist < a) { b = a; a = dist; ia = j; }
        else if (dist < b) { b = dist; }
    }
    *d1 = a; *d2 = b; *arg = ia;
    return ORC_OK;
}
