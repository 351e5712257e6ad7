/*
 * rls - adaptive-sampling hot path on one MI355X (gfx950): C ABI.
 *
 * The calls follow the paper's statement of the adaptive-sampling step
 * (Sec. 4.2, Algorithm 1) and of the cost-model query that precedes it
 * (Sec. 4.1, "Reward formulation" / "Learning procedure"):
 *
 *   rls_gbt_score       predicted fitness of every configuration of a trajectory
 *   rls_kmeans_sweep    k-means(s_Theta, k) for every k of a range: centroids, clusters, loss
 *   rls_pick_knee       the knee test on the loss curve (host, scalar)
 *   rls_kmeans_sweep_until_knee  the same loop with Algorithm 1's early exit at the knee
 *   rls_snap_to_valid   NextSamples = Centroids, as valid configurations
 *   rls_knob_modes      mode(s_Theta), dimension by dimension
 *   rls_replace_visited samples already in v_Theta give way to mode(s_Theta)
 *   rls_apply_actions   the search agent's configuration updater (producer of the trajectory)
 *
 * Conventions
 *   - Plain C. Every call returns an int32_t status: RLS_OK or a negative RLS_ERR_* code.
 *   - Pointers named *_dev are device (HBM) pointers owned by the caller; all others are host
 *     pointers.  The library never allocates or frees device memory: scratch space comes in
 *     through `workspace_dev`, sized by the matching *_workspace_bytes query.
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue kernels on it and return
 *     without synchronising; outputs are valid once the stream has drained.  The one exception,
 *     rls_kmeans_sweep_until_knee, says so.  Such a call may be recorded into a HIP graph by the
 *     caller (kernels only: nothing is allocated, copied to the host or cleared with a memset node;
 *     call it once outside the capture first, which sets the kernels' launch attributes).
 *   - Results do not depend on the run: labels, centroids, configurations and scores are exact or
 *     summed in a fixed order, and so are the reported losses.
 *   - Matrices are row-major fp32 with an explicit leading dimension in elements.
 *   - Argument errors are detected on the host before anything is enqueued.  Conditions that
 *     only the data can reveal (see rls_kmeans_sweep) are reported through `status_dev`.
 *   - Limits: 1 <= d <= RLS_MAX_D, k_max <= RLS_MAX_K, tree depth <= RLS_MAX_DEPTH,
 *     N <= RLS_MAX_N, batch <= RLS_MAX_BATCH; rls_kmeans_sweep also needs ldx <= RLS_MAX_LDX.
 */
#ifndef RLS_H
#define RLS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RLS_OK 0
#define RLS_ERR_INVALID_ARG (-1)   /* a size, range or limit is violated */
#define RLS_ERR_NULL (-2)          /* a required pointer is NULL */
#define RLS_ERR_SHAPE (-3)         /* shapes disagree (forest features vs d, ldx < d, ...) */
#define RLS_ERR_WORKSPACE (-4)     /* workspace missing, misaligned (256 B) or too small */
#define RLS_ERR_HIP (-5)           /* a HIP runtime call failed; see rls_last_hip_error() */
#define RLS_ERR_NOT_IMPLEMENTED (-6)

#define RLS_MAX_D 32
#define RLS_MAX_K 128
#define RLS_MAX_DEPTH 12
#define RLS_MAX_N (1LL << 26)
#define RLS_MAX_BATCH 1024
#define RLS_MAX_LDX (1 << 24)       /* leading dimension of X accepted by rls_kmeans_sweep (elements) */

/* bits of *status_dev written by rls_kmeans_sweep (0 = clean) */
#define RLS_STATUS_NONFINITE 1     /* X holds an infinity or NaN */
#define RLS_STATUS_RANGE 2         /* a feature column is too wide for exact fixed-point sums */

int32_t rls_version(void);
const char *rls_error_string(int32_t code);
/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
int32_t rls_last_hip_error(void);

/*
 * Boosted-tree cost model (Sec. 4.1: the estimate of the cost model is the surrogate reward;
 * the whole trajectory is scored after each episode).  The paper names the model family only;
 * the layout here is: `n_trees` complete binary trees of depth `depth` in level order, node n
 * having children 2n+1 (taken when x[feat] < thr) and 2n+2 (otherwise, NaN included).
 * All three arrays are borrowed device pointers.
 */
typedef struct {
    int32_t n_trees;
    int32_t depth;             /* 1..RLS_MAX_DEPTH */
    int32_t n_features;        /* must equal d of the matrix scored */
    float base;                /* added before the first tree */
    const int32_t *feat_dev;   /* [n_trees][2^depth - 1] feature index of each internal node */
    const float *thr_dev;      /* [n_trees][2^depth - 1] threshold of each internal node */
    const float *leaf_dev;     /* [n_trees][2^depth] leaf values */
} rls_forest;

/*
 * score_dev[i] = base + sum_t leaf_t(walk_t(X[i])), added in fp32 in tree order t = 0, 1, ...
 *   X_dev      [N][ldx] fp32, first d columns used
 *   score_dev  [N] fp32 (written)
 * A feature index outside [0, d) is read as the nearest valid column (0 or d - 1): the forest lives in device
 * memory, which the host checks never read, and the walk must not leave the row.
 */
int32_t rls_gbt_score(const rls_forest *forest, const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                      float *score_dev, void *stream);

/*
 * `batch` independent knob spaces, each with its own forest (host array of `batch` structs) and
 * its own N x d block of X: space b reads X_dev + b * x_batch_stride and writes score_dev + b * N.
 */
int32_t rls_gbt_score_batched(const rls_forest *forests, int32_t batch, const float *X_dev, int64_t N,
                              int32_t d, int64_t ldx, int64_t x_batch_stride, float *score_dev, void *stream);

/*
 * k-means++ seeding chain (D^2 sampling) of k_max centres drawn with the counter-based
 * generator SplitMix64(seed + (j+1) * 0x9E3779B97F4A7C15), top 53 bits as a uniform in [0,1).
 * The paper does not fix the initialisation of k-means; a run with k clusters starts from
 * the first k centres of this chain.
 *   init_idx_dev  [k_max] int64 row indices (written)
 *   workspace     rls_kmeans_sweep_workspace_bytes(N, d, k_max, k_max, 1) bytes suffice
 */
int32_t rls_kmeanspp_chain(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_max, uint64_t seed,
                           int64_t *init_idx_dev, void *workspace_dev, int64_t workspace_bytes, void *stream);

/* Bytes of workspace rls_kmeans_sweep[_batched] needs (a multiple of 256), or a negative RLS_ERR_* code. */
int64_t rls_kmeans_sweep_workspace_bytes(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t batch);

/*
 * The loop over k of Algorithm 1 (Sec. 4.2) without its early break: Lloyd's k-means for
 * every k in [k_min, k_max], each run independent and started from the first k centres of
 * one seeding chain, `iters` rounds of (assign, update) and a final assignment.
 *   - distance: squared Euclidean on the fp32 rows as given; ties go to the lowest centroid index
 *   - centroid: fp32( fp64(exact sum of the members) / count ); a cluster without members keeps
 *     its centroid
 *   - loss (inertia): sum of squared distances to the assigned centroid, against the returned
 *     centroids, accumulated in fp64
 * Arguments
 *   X_dev             [N][ldx] fp32
 *   k_min..k_max      inclusive, 1 <= k_min <= k_max <= min(N, RLS_MAX_K)
 *   iters             >= 0
 *   seed              used only when init_idx_dev is NULL
 *   init_idx_dev      [k_max] int64 row indices of the initial centres, or NULL to draw the chain
 *   labels_dev        [n_k][N] int32 (n_k = k_max-k_min+1), or NULL
 *   centroids_dev     packed fp32: run k starts at element d * sum_{k_min <= k' < k} k'; sum(k)*d floats
 *   inertia_dev       [n_k] fp64
 *   inertia_trace_dev [n_k][iters+1] fp64 loss of assignment t against the centroids it used, or NULL
 *   status_dev        one int32 (written): 0, or RLS_STATUS_* bits when the data breaks a
 *                     precondition, in which case all other outputs are unspecified.  Exact sums
 *                     need, per feature column, the lowest set bit of every value to lie at most
 *                     79 binary places below the highest set bit of the column.
 *   workspace_dev     256-byte aligned, at least rls_kmeans_sweep_workspace_bytes(...) bytes
 */
int32_t rls_kmeans_sweep(const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                         int32_t k_min, int32_t k_max, int32_t iters, uint64_t seed,
                         const int64_t *init_idx_dev, int32_t *labels_dev, float *centroids_dev,
                         double *inertia_dev, double *inertia_trace_dev, int32_t *status_dev,
                         void *workspace_dev, int64_t workspace_bytes, void *stream);

/*
 * rls_kmeans_sweep for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, results and status bits, but the workspace is a fixed
 * array of RLS_STATIC_WORKSPACE_BYTES inside the library's device image (each GPU the library runs on holds its
 * own copy until the process ends).  The call allocates nothing and frees nothing.
 *   - RLS_ERR_WORKSPACE when rls_kmeans_sweep_workspace_bytes(N, d, k_min, k_max, 1) exceeds
 *     RLS_STATIC_WORKSPACE_BYTES (nothing is enqueued); that query tells beforehand whether a shape fits.
 *   - All calls on one GPU share that GPU's array: two such sweeps that overlap in time on one GPU (different
 *     streams or host threads) race.  Successive calls on one stream are fine; every call initialises the parts
 *     of the array it reads.
 */
#define RLS_STATIC_WORKSPACE_BYTES (64 << 20)
int32_t rls_kmeans_sweep_static(const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                                int32_t k_min, int32_t k_max, int32_t iters, uint64_t seed,
                                const int64_t *init_idx_dev, int32_t *labels_dev, float *centroids_dev,
                                double *inertia_dev, double *inertia_trace_dev, int32_t *status_dev, void *stream);

/*
 * `batch` independent spaces of equal shape in one launch sequence.  Space b reads
 * X_dev + b * x_batch_stride, uses seeds[b] (host array) or init_idx_dev + b * k_max, and writes
 * block b of every output: labels [batch][n_k][N], centroids [batch][sum(k)*d], inertia [batch][n_k],
 * trace [batch][n_k][iters+1], status [batch].
 */
int32_t rls_kmeans_sweep_batched(int32_t batch, const float *X_dev, int64_t N, int32_t d, int64_t ldx,
                                 int64_t x_batch_stride, int32_t k_min, int32_t k_max, int32_t iters,
                                 const uint64_t *seeds, const int64_t *init_idx_dev, int32_t *labels_dev,
                                 float *centroids_dev, double *inertia_dev, double *inertia_trace_dev,
                                 int32_t *status_dev, void *workspace_dev, int64_t workspace_bytes, void *stream);

/*
 * Algorithm 1's loop as it is written: k-means for k = k_min, k_min + 1, ... until the knee test fires, then stop.
 * The k are taken k_wave at a time (one sweep per wave, its k side by side as in rls_kmeans_sweep); after each wave
 * this call SYNCHRONISES `stream`, copies the wave's losses to inertia_host and applies the test of rls_pick_knee in
 * k order.  The outputs for the k that were computed equal those of rls_kmeans_sweep over the whole range, and
 * *k_out equals rls_pick_knee on the whole curve: runs for different k do not depend on each other.
 *   k_wave        >= 1; a multiple of 8 keeps the MFMA tiles full.  The k of a wave share each read of the points, and
 *                 the waves of a call share the column statistics and the prepared copy of the points: larger waves
 *                 cost less per k, smaller ones stop closer behind the knee
 *   seed / init_idx_dev  as rls_kmeans_sweep (the chain is extended wave by wave)
 *   labels_dev    [k_max-k_min+1][N] or null; centroids_dev, inertia_dev as rls_kmeans_sweep; only the first
 *                 *n_done_out runs are written
 *   inertia_host  [k_max-k_min+1] fp64 (host), first *n_done_out entries written
 *   k_out         the chosen k (k_max when the test never fires; 0 when *status_dev != 0)
 *   n_done_out    how many k were computed (a whole number of waves, or all)
 * Workspace: rls_kmeans_sweep_until_knee_workspace_bytes.
 */
int64_t rls_kmeans_sweep_until_knee_workspace_bytes(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t k_wave);
int32_t rls_kmeans_sweep_until_knee(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_min, int32_t k_max,
                                    int32_t k_wave, int32_t iters, uint64_t seed, const int64_t *init_idx_dev,
                                    double knee_const, int32_t *labels_dev, float *centroids_dev, double *inertia_dev,
                                    double *inertia_host, int32_t *k_out, int32_t *n_done_out, int32_t *status_dev,
                                    void *workspace_dev, int64_t workspace_bytes, void *stream);

/*
 * Knee of the loss curve (Algorithm 1): with PreviousLoss = infinity, walk k upward and stop at the
 * first k with knee_const * inertia[k] > PreviousLoss; that k (whose centroids Algorithm 1 has
 * already assigned when the test fires) is returned, or k_max when the test never fires.
 * Pure host function; inertia_host is [k_max-k_min+1] fp64.  The paper names the constant without
 * giving its value, so it is an argument.
 */
int32_t rls_pick_knee(const double *inertia_host, int32_t k_min, int32_t k_max, double knee_const, int32_t *k_out);

/*
 * Knob domains of one design space (Sec. 2.2: the space is the product of the knob domains):
 * knob j owns values_dev[offsets[j] .. offsets[j+1]) and reads feature column j.
 */
typedef struct {
    int32_t n_knobs;             /* 1..d */
    const int32_t *offsets_dev;  /* [n_knobs+1], strictly increasing */
    const float *values_dev;     /* [offsets[n_knobs]] */
} rls_knob_domains;

/*
 * NextSamples = Centroids (Algorithm 1): each centroid becomes a valid configuration by taking,
 * knob by knob, the index of the nearest domain value (|c - v| compared in fp64, ties to the lower index).
 *   centroids_dev [k][ldc] fp32;  cfg_dev [k][n_knobs] int32 domain indices (written)
 */
int32_t rls_snap_to_valid(const float *centroids_dev, int32_t k, int32_t d, int64_t ldc,
                          const rls_knob_domains *domains, int32_t *cfg_dev, void *stream);

/* Space b: centroids_dev + b * c_batch_stride, domains[b] (host array), cfg_dev + b * k * n_knobs. */
int32_t rls_snap_to_valid_batched(int32_t batch, const float *centroids_dev, int32_t k, int32_t d, int64_t ldc,
                                  int64_t c_batch_stride, const rls_knob_domains *domains, int32_t *cfg_dev,
                                  void *stream);

/*
 * mode(s_Theta) of Algorithm 1, which Sec. 4.2 describes as the configuration "generated from modes of each
 * dimension": for every knob j, the domain index that most rows of the trajectory take, a row's value in
 * knob j being the domain entry nearest to its coordinate j (same rule as rls_snap_to_valid: |x - v| in
 * fp64, ties to the lower index).  Equally frequent entries: the lower index.
 *   X_dev        [N][ldx] fp32, N <= 2^26
 *   mode_cfg_dev [n_knobs] int32 (written)
 *   hist_dev     [offsets[n_knobs]] int32 counts of every domain entry, laid out like values_dev; used as
 *                scratch and left holding the counts.  At most RLS_MAX_DOMAIN_VALUES entries in total.
 * domains->offsets_dev and values_dev are device arrays; n_total_values = offsets[n_knobs] is passed by the
 * caller (the library does not read device memory on the host).
 */
#define RLS_MAX_DOMAIN_VALUES 8192
int32_t rls_knob_modes(const float *X_dev, int64_t N, int32_t d, int64_t ldx, const rls_knob_domains *domains,
                       int32_t n_total_values, int32_t *mode_cfg_dev, int32_t *hist_dev, void *stream);

/*
 * The last loop of Algorithm 1: a sample that is already among the visited configurations v_Theta is
 * replaced by mode(s_Theta).  Configurations are rows of n_knobs domain indices.
 *   cfg_dev      [k][n_knobs] int32, updated in place; 1 <= k <= 65535
 *   visited_dev  [n_visited][n_knobs] int32 (may be null when n_visited == 0)
 *   mode_cfg_dev [n_knobs] int32
 *   replaced_dev [k] int32 (written): 1 where the row was replaced
 * The replacement is not checked against v_Theta again (the paper's loop does not).
 */
int32_t rls_replace_visited(int32_t *cfg_dev, int32_t k, int32_t n_knobs, const int32_t *visited_dev,
                            int64_t n_visited, const int32_t *mode_cfg_dev, int32_t *replaced_dev, void *stream);

/*
 * Configuration updater of the search agent (Sec. 4.1, "Action space", "Learning procedure"): an action is one
 * direction per dimension (-1 decrement, 0 stay, +1 increment); applying it to a configuration gives the next one
 * of the trajectory.  A step that would leave a knob's domain stays at the border (the paper does not say).
 *   cfg_dev      [m][n_knobs] int32 domain indices (values outside a domain are first brought to its border)
 *   action_dev   [m][n_knobs] int8 (values beyond +-1 count as +-1)
 *   cfg_out_dev  [m][n_knobs] int32 (written; may be cfg_dev)
 *   features_dev [m][ldf] fp32 or null: the first n_knobs columns receive the domain values of the new
 *                configurations, the form in which rls_gbt_score is queried for a whole trajectory
 */
int32_t rls_apply_actions(const int32_t *cfg_dev, const int8_t *action_dev, int64_t m, const rls_knob_domains *domains,
                          int32_t *cfg_out_dev, float *features_dev, int64_t ldf, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RLS_H */
