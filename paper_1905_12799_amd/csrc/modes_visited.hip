// The last loop of Algorithm 1 of the paper: samples that were visited before are replaced by mode(s_Theta),
// the configuration made of the mode of each dimension of the trajectory (Sec. 4.2).
//
// knob_hist_kernel   every workgroup keeps the domain values and a histogram over all domain entries in LDS;
//                    a thread takes whole rows of the trajectory, finds for every knob the nearest domain entry
//                    (|x - v| in fp64, first minimum wins, as in the snap kernel; a bisection when the knob's
//                    entries are sorted) and counts it with an integer LDS atomic, or per entry with a wave
//                    ballot when the knob has only a few; the workgroup then adds its counts to the global
//                    histogram (integer atomics: the result does not depend on the order).
// knob_mode_kernel   one thread per knob: first maximum of its slice of the histogram.
// visited_scan_kernel / visited_apply_kernel  workgroups compare one sample with a slice of the visited rows and
//                    flag it; flagged samples are then overwritten with the mode.
#include "rls_internal.h"

namespace rls {

namespace {

constexpr int kHistThreads = 256;
constexpr int kMaxKnobs = RLS_MAX_D;

__global__ void fill_zero_kernel(int32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// nearest entry of vals[lo, hi) to x: |x - v| in fp64, the first minimum wins.  `sorted`: the slice is
// non-decreasing, so two probes around the lower bound decide; otherwise the slice is scanned.
__device__ inline int nearest_entry(const float *vals, int lo, int hi, float xf, bool sorted)
{
    const double x = (double)xf;
    if (!sorted) {
        double best = INFINITY;
        int arg = lo;
        for (int v = lo; v < hi; ++v) {
            const double gap = fabs(x - (double)vals[v]);
            if (gap < best) { best = gap; arg = v; }
        }
        return arg;
    }
    int a = lo, b = hi;                       // first entry >= x
    while (a < b) {
        const int m = (a + b) >> 1;
        if (vals[m] < xf) a = m + 1; else b = m;
    }
    int arg = a < hi ? a : hi - 1;
    if (a > lo && a < hi) {
        // entry below against entry at or above: the lower index wins a tie
        if (fabs(x - (double)vals[a - 1]) <= fabs(x - (double)vals[a])) arg = a - 1;
    }
    while (arg > lo && vals[arg - 1] == vals[arg]) --arg;     // equal entries: the first of them
    return arg;
}

__global__ void __launch_bounds__(kHistThreads) knob_hist_kernel(const float *__restrict__ X, int64_t N, int64_t ldx,
                                                                  DomainArgs dm, int n_total, int32_t *__restrict__ hist)
{
    extern __shared__ __align__(16) unsigned char smem[];
    float *vals = reinterpret_cast<float *>(smem);                 // [n_total]
    int *cnt = reinterpret_cast<int *>(vals + n_total);            // [n_total]
    __shared__ int offs[kMaxKnobs + 1];
    __shared__ int unsorted[kMaxKnobs];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int e = tid; e < n_total; e += kHistThreads) { vals[e] = dm.values[e]; cnt[e] = 0; }
    if (tid <= dm.n_knobs) offs[tid] = dm.offsets[tid];
    if (tid < kMaxKnobs) unsorted[tid] = 0;
    __syncthreads();
    for (int e = tid; e + 1 < n_total; e += kHistThreads) {
        if (vals[e + 1] < vals[e]) {
            // a descent inside one knob's slice (not across a boundary) marks that knob as unsorted
            for (int j = 0; j < dm.n_knobs; ++j)
                if (e >= offs[j] && e + 1 < offs[j + 1]) unsorted[j] = 1;
        }
    }
    __syncthreads();

    // whole waves enter the loop together (the ballots below need every lane of a wave)
    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    const int64_t rounds = (N + stride - 1) / stride;
    for (int64_t r = 0; r < rounds; ++r) {
        const int64_t i = r * stride + (int64_t)blockIdx.x * kHistThreads + tid;
        const bool valid = i < N;
        const float *row = X + (valid ? i : 0) * ldx;
        // the knob columns of the row eight at a time: all eight loads are out before the first search starts
        for (int j0 = 0; j0 < dm.n_knobs; j0 += 8) {
            float xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xv[u] = row[min(j0 + u, dm.n_knobs - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = j0 + u;
                if (j >= dm.n_knobs) break;              // same for every lane
                const int lo = offs[j], hi = offs[j + 1];
                const int arg = valid ? nearest_entry(vals, lo, hi, xv[u], unsorted[j] == 0) : -1;
                if (hi - lo <= 8) {
                    // few entries: most lanes would hit the same counters; count per entry with a ballot instead
                    for (int v = lo; v < hi; ++v) {
                        const int c = __popcll(__ballot(arg == v));
                        if (lane == 0 && c) atomicAdd(&cnt[v], c);
                    }
                } else if (valid) {
                    atomicAdd(&cnt[arg], 1);
                }
            }
        }
    }
    __syncthreads();
    for (int e = tid; e < n_total; e += kHistThreads)
        if (cnt[e] != 0) atomicAdd(&hist[e], cnt[e]);
}

__global__ void knob_mode_kernel(DomainArgs dm, const int32_t *__restrict__ hist, int32_t *__restrict__ mode_cfg)
{
    const int j = threadIdx.x;
    if (j >= dm.n_knobs) return;
    const int lo = dm.offsets[j], hi = dm.offsets[j + 1];
    int arg = lo;
    for (int v = lo + 1; v < hi; ++v)
        if (hist[v] > hist[arg]) arg = v;
    mode_cfg[j] = arg - lo;
}

// grid (slices of the visited rows, samples): a workgroup compares one sample with its slice of v_Theta
__global__ void __launch_bounds__(kHistThreads) visited_scan_kernel(const int32_t *__restrict__ cfg, int n_knobs,
                                                                     const int32_t *__restrict__ visited, int64_t n_visited,
                                                                     int64_t slice, int32_t *__restrict__ replaced)
{
    __shared__ int mine[kMaxKnobs];
    const int i = blockIdx.y, tid = threadIdx.x;
    if (tid < n_knobs) mine[tid] = cfg[(int64_t)i * n_knobs + tid];
    __syncthreads();
    const int64_t v0 = (int64_t)blockIdx.x * slice, v1 = min(n_visited, v0 + slice);
    int hit = 0;
    for (int64_t v = v0 + tid; v < v1; v += kHistThreads) {
        const int32_t *row = visited + v * n_knobs;
        int same = 1;
        for (int j = 0; j < n_knobs; ++j) same &= (row[j] == mine[j]) ? 1 : 0;
        hit |= same;
    }
    if (__ballot(hit != 0) != 0ull && (tid & 63) == 0) atomicOr(&replaced[i], 1);
}

// one thread per (sample, knob): visited samples take the mode
__global__ void visited_apply_kernel(int32_t *__restrict__ cfg, int k, int n_knobs, const int32_t *__restrict__ mode_cfg,
                                     const int32_t *__restrict__ replaced)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= k * n_knobs) return;
    if (replaced[e / n_knobs]) cfg[e] = mode_cfg[e % n_knobs];
}

// Configuration updater of the search agent (Sec. 4.1 of the paper): one thread per (configuration, knob) adds the
// direction to the domain index and holds it at the domain's borders; optionally writes the knob's value as feature.
// (cfg and cfg_out may be the same array: neither is declared restrict; a thread reads its element before it writes it)
__global__ void apply_actions_kernel(const int32_t *cfg, const signed char *__restrict__ action, int64_t m,
                                     DomainArgs dm, int32_t *cfg_out, float *__restrict__ features, int64_t ldf)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= m * dm.n_knobs) return;
    const int64_t i = e / dm.n_knobs;
    const int j = (int)(e % dm.n_knobs);
    const int lo = dm.offsets[j], size = dm.offsets[j + 1] - lo;
    int a = action[e];
    a = a < -1 ? -1 : (a > 1 ? 1 : a);                 // directions only
    int v = cfg[e];
    v = v < 0 ? 0 : (v > size - 1 ? size - 1 : v);     // a configuration outside its domain is brought inside first
    v += a;
    v = v < 0 ? 0 : (v > size - 1 ? size - 1 : v);
    cfg_out[e] = v;
    if (features) features[i * ldf + j] = dm.values[lo + v];
}

}  // namespace

hipError_t launch_knob_modes(const float *X, int64_t N, int64_t ldx, const DomainArgs &dm, int32_t n_total,
                             int32_t *mode_cfg, int32_t *hist, hipStream_t s)
{
    hipLaunchKernelGGL(fill_zero_kernel, dim3((n_total + 255) / 256), dim3(256), 0, s, hist, (int)n_total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // enough workgroups to fill the chip a few times; each row costs n_knobs short scans
    int64_t blocks = (N + kHistThreads * 4 - 1) / (kHistThreads * 4);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    const size_t lds = (size_t)n_total * 8;
    hipLaunchKernelGGL(knob_hist_kernel, dim3((unsigned)blocks), dim3(kHistThreads), lds, s, X, N, ldx, dm, (int)n_total, hist);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(knob_mode_kernel, dim3(1), dim3(64), 0, s, dm, hist, mode_cfg);
    return hipGetLastError();
}

hipError_t launch_replace_visited(int32_t *cfg, int32_t k, int32_t n_knobs, const int32_t *visited, int64_t n_visited,
                                  const int32_t *mode_cfg, int32_t *replaced, hipStream_t s)
{
    hipLaunchKernelGGL(fill_zero_kernel, dim3((k + 255) / 256), dim3(256), 0, s, replaced, (int)k);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_visited == 0) return e;
    // slices of at least 4096 rows, at most ~1024 workgroups in all
    int64_t slices = (n_visited + 4095) / 4096;
    const int64_t cap = (1024 + k - 1) / k;
    if (slices > cap) slices = cap;
    if (slices < 1) slices = 1;
    const int64_t slice = (n_visited + slices - 1) / slices;
    hipLaunchKernelGGL(visited_scan_kernel, dim3((unsigned)slices, (unsigned)k), dim3(kHistThreads), 0, s, cfg, (int)n_knobs,
                       visited, n_visited, slice, replaced);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(visited_apply_kernel, dim3((k * n_knobs + 255) / 256), dim3(256), 0, s, cfg, (int)k, (int)n_knobs,
                       mode_cfg, replaced);
    return hipGetLastError();
}

hipError_t launch_apply_actions(const int32_t *cfg, const signed char *action, int64_t m, const DomainArgs &dm,
                                int32_t *cfg_out, float *features, int64_t ldf, hipStream_t s)
{
    const int64_t total = m * dm.n_knobs;
    hipLaunchKernelGGL(apply_actions_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, cfg, action, m, dm, cfg_out,
                       features, ldf);
    return hipGetLastError();
}

}  // namespace rls
