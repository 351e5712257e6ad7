// Internal declarations shared by the host entry points and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rls.h"
#include "rls_bench.h"

namespace rls {

// last failing hipError_t on this thread
void set_hip_error(hipError_t e);

#define RLS_HIP_TRY(expr)                      \
    do {                                       \
        hipError_t rls_e_ = (expr);            \
        if (rls_e_ != hipSuccess) {            \
            ::rls::set_hip_error(rls_e_);      \
            return RLS_ERR_HIP;                \
        }                                      \
    } while (0)

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// ---------------------------------------------------------------------------------------------
// Sweep plan: how the runs (one per k) of a sweep are packed into workgroup-sized groups.
//
// An MFMA tile has 32 centroid rows = 8 quads of 4 rows.  Quad `slot` (0..7) of every tile of a
// group belongs to one run for the whole group, so the running (best, second best) of a point
// never leaves its lane.  A group holds R = 8 / S runs, each owning S slots.
// Centroid j of run r sits in tile (j/4)/S, slot r*S + (j/4)%S, row-in-quad j%4.
struct GroupDesc {
    int16_t run0;      // index of the first run (k = k_min + run0)
    int16_t n_runs;    // real runs in this group (<= 8 / S)
    int16_t S;         // slots per run: 1, 2, 4 or 8
    int16_t n_tiles;   // 32-row tiles
    int16_t copies;    // copies of the LDS accumulators (a power of two up to 16)
    int16_t lab0;      // run slots (8 / S each) of all earlier groups: where this group's label bytes begin, in units of N rounded up to 16
    int32_t tile0;     // tiles of all earlier groups (offset of this group's operand block)
};

constexpr int kMaxGroups = 128;

struct SweepPlan {
    int32_t n_groups;
    int32_t n_runs;      // k_max - k_min + 1
    int32_t k_min;
    int32_t total_tiles;
    int32_t lab_slots;   // sum over the groups of their 8 / S run slots
    int32_t total_rows;  // sum of k over the runs
    int32_t n_chunks;    // point chunks per group
    int32_t chunk_len;   // points per chunk (multiple of the tile size)
    int32_t chunk_block; // chunks per block of the step kernel's workgroup order (all groups of a block of chunks, then the next block)
    int32_t dp;          // padded feature count: 8, 16 or 32
    GroupDesc g[kMaxGroups];
    uint8_t sched[kMaxGroups];   // launch order: group indices by falling cost
};

// rows of runs k_min .. k_min+run-1
__host__ __device__ inline int32_t rows_before(int32_t k_min, int32_t run) {
    return run * k_min + run * (run - 1) / 2;
}

struct LloydGeometry {
    int threads;      // workgroup size
    int tile_points;  // points per tile
    int lds_budget;   // bytes of LDS one workgroup may use
};
LloydGeometry lloyd_geometry(int dp);
int padded_d(int d);
// LDS bytes of a group: operand tiles + centroid copy + exact-sum accumulators + fixed part
int64_t lloyd_group_lds_bytes(int dp, int d, int n_tiles, int real_rows, int copies);
// `batch`: spaces swept by the same launches (sizes the chunks so that the whole batch gives ~512 workgroups)
int32_t make_sweep_plan(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t batch, SweepPlan *plan);

// Workspace carving for one sweep (all offsets in bytes from the workspace base, per batch element
// unless noted).  Filled by sweep_layout().
struct SweepLayout {
    int64_t colstat_part;   // per-block partial column statistics
    int64_t colinfo;        // mean[32] fp32, shift[32] int32, wide[33] int32
    int64_t chain;          // int64 [k_max] seeding chain
    int64_t mind;           // fp64 [N] squared distance to the nearest chosen centre
    int64_t bsum;           // fp64 [seed blocks] block sums of mind
    int64_t near;           // uint8 [N] chain position of the nearest chosen centre
    int64_t seedthr;        // fp64 [k_max] per chosen centre: the bound below which a point's distance cannot improve
    int64_t opA;            // per 32-row tile: fp16 pieces of the centred, -2-scaled centroids and the bf16 bias slot, in MFMA operand order
    int64_t cnmax;          // fp32 [n_runs][parts of a run] maximum of cn over the centroids of a part
    int64_t psum;           // int64 [n_chunks][total_rows][d] per-chunk changes of the fixed-point sums
    int64_t pcnt;           // int32 [n_chunks][total_rows] per-chunk changes of the member counts
    int64_t pj;             // fp64 [n_chunks][n_runs] partial losses
    int64_t losum;          // int64 [total_rows][d] low-order fixed-point sums of wide columns (running)
    int64_t tot;            // int64 [total_rows][d][2] running 128-bit fixed-point sums (hi, lo)
    int64_t totcnt;         // int64 [total_rows][d] running member counts (one copy per feature)
    int64_t prev;           // uint8 per group [N rounded up to 16][8 / S]: label of every point in the last round (0xff: none yet)
    int64_t log;            // uint64 [groups * chunks][waves][512] rings of moved-pair records, one per wave of the step kernel
    int64_t xp;             // prepared copy of the points: per block of 32, the matrix operands and squared norms (kmeans_lloyd.hip)
    int64_t per_batch;      // bytes per batch element (multiple of 256)
    int64_t total;          // per_batch * batch
    int32_t seed_blocks;
    int32_t stat_blocks;
};
void sweep_layout(const SweepPlan &plan, int64_t N, int32_t d, int32_t k_max, int32_t batch, SweepLayout *L);

constexpr int kSeedBlock = 1024;   // points per block of the seeding kernels
constexpr int kStatBlocks = 256;   // blocks of the column-statistics kernel

// ---------------------------------------------------------------------------------------------
// kernel launchers (each enqueues on `s` and returns a HIP status)
struct ForestArgs {
    int32_t n_trees, depth;
    float base;
    const int32_t *feat;
    const float *thr;
    const float *leaf;
};
hipError_t launch_gbt_score(const ForestArgs *forests_host, int32_t batch, const float *X, int64_t N, int32_t d,
                            int64_t ldx, int64_t x_batch_stride, float *score, hipStream_t s);

struct DomainArgs {
    int32_t n_knobs;
    const int32_t *offsets;
    const float *values;
};
hipError_t launch_snap(const DomainArgs *domains_host, int32_t batch, const float *C, int32_t k, int32_t d, int64_t ldc,
                       int64_t c_batch_stride, int32_t *cfg, hipStream_t s);

hipError_t launch_knob_modes(const float *X, int64_t N, int64_t ldx, const DomainArgs &dm, int32_t n_total,
                             int32_t *mode_cfg, int32_t *hist, hipStream_t s);
hipError_t launch_replace_visited(int32_t *cfg, int32_t k, int32_t n_knobs, const int32_t *visited, int64_t n_visited,
                                  const int32_t *mode_cfg, int32_t *replaced, hipStream_t s);

hipError_t launch_apply_actions(const int32_t *cfg, const signed char *action, int64_t m, const DomainArgs &dm,
                                int32_t *cfg_out, float *features, int64_t ldf, hipStream_t s);

hipError_t launch_seed_chain(const float *X, int64_t N, int32_t d, int64_t ldx, int64_t x_batch_stride, int32_t batch,
                             int32_t k_max, const uint64_t *seeds_host, int64_t *chain, int64_t chain_batch_stride,
                             char *ws, const SweepLayout &L, hipStream_t s, int32_t j_begin = 0);

struct SweepArgs {
    const float *X;
    int64_t N;
    int32_t d;
    int64_t ldx;
    int64_t x_batch_stride;
    int32_t batch;
    int32_t iters;
    const int64_t *init_idx;      // [batch][k_max]
    int64_t init_batch_stride;
    int32_t *labels;              // [batch][n_runs][N] or null
    float *centroids;             // [batch][total_rows * d]
    double *inertia;              // [batch][n_runs]
    double *trace;                // [batch][n_runs][iters+1] or null
    int32_t *status;              // [batch]
    char *ws;                     // workspace base
    // A sweep over the same rows with the same workspace has run before (the waves of a sweep that stops at the knee):
    // the column information, and the prepared copy of the points, are still in place and are not made again.
    int32_t reuse_colstats;
    int32_t reuse_prepared;
};
// benchmark timing of the Lloyd step kernel (see rls_bench.h)
bool profile_enabled();
hipError_t profile_mark(hipStream_t s, bool begin);

hipError_t launch_sweep(const SweepPlan &plan, const SweepLayout &L, const SweepArgs &a, hipStream_t s);
// whether the rounds after the first of such a sweep read the prepared copy of the points
bool sweep_uses_prepared(const SweepPlan &plan, int32_t iters, bool trace);

}  // namespace rls
