// Centroids -> valid configurations ("NextSamples = Centroids", Algorithm 1 of the paper).
// One thread per (centroid, knob): scan the knob's domain for the value nearest to the centroid's
// coordinate, comparing |c - v| in fp64 with a strict "<" so that the first minimum (lower index) wins.
#include "rls_internal.h"

namespace rls {

namespace {

constexpr int kSnapBatch = 64;   // spaces per launch (domain descriptors travel as kernel arguments)

struct SnapArgs {
    DomainArgs dom[kSnapBatch];
};

__global__ void snap_kernel(SnapArgs a, const float *__restrict__ C, int k, int64_t ldc, int64_t c_batch_stride,
                            int32_t *__restrict__ cfg, int n_knobs_out)
{
    const DomainArgs dm = a.dom[blockIdx.y];
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= k * dm.n_knobs) return;
    const int i = e / dm.n_knobs, j = e % dm.n_knobs;
    const double c = (double)C[(int64_t)blockIdx.y * c_batch_stride + (int64_t)i * ldc + j];
    const int lo = dm.offsets[j], hi = dm.offsets[j + 1];
    double best = INFINITY;
    int arg = 0;
    for (int v = lo; v < hi; ++v) {
        const double gap = fabs(c - (double)dm.values[v]);
        if (gap < best) { best = gap; arg = v - lo; }
    }
    cfg[((int64_t)blockIdx.y * k + i) * n_knobs_out + j] = arg;
}

}  // namespace

hipError_t launch_snap(const DomainArgs *domains_host, int32_t batch, const float *C, int32_t k, int32_t d, int64_t ldc,
                       int64_t c_batch_stride, int32_t *cfg, hipStream_t s)
{
    (void)d;
    for (int32_t b0 = 0; b0 < batch; b0 += kSnapBatch) {
        const int nb = batch - b0 < kSnapBatch ? batch - b0 : kSnapBatch;
        SnapArgs a;
        int max_knobs = 0;
        for (int b = 0; b < nb; ++b) {
            a.dom[b] = domains_host[b0 + b];
            if (a.dom[b].n_knobs > max_knobs) max_knobs = a.dom[b].n_knobs;
        }
        for (int b = nb; b < kSnapBatch; ++b) a.dom[b] = a.dom[0];
        const int n_knobs = domains_host[b0].n_knobs;   // all spaces of a batch share n_knobs (checked by the caller)
        const int threads = 128;
        const unsigned gx = (unsigned)((k * max_knobs + threads - 1) / threads);
        hipLaunchKernelGGL(snap_kernel, dim3(gx, nb), dim3(threads), 0, s, a, C + (int64_t)b0 * c_batch_stride, (int)k, ldc,
                           c_batch_stride, cfg + (int64_t)b0 * k * n_knobs, n_knobs);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rls
