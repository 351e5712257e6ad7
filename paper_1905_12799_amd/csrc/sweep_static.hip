// rls_kmeans_sweep_static: rls_kmeans_sweep for callers that cannot allocate device memory.  The workspace that
// rls_kmeans_sweep takes from its caller is a fixed array in this library's device image instead; everything else
// (argument checks, plan, kernels, results) is the code path of rls_kmeans_sweep.
#include <mutex>

#include "rls_internal.h"

namespace {

// The workspace, one copy per GPU the library runs on, held until the process ends.  In host code this name is
// only a handle for hipGetSymbolAddress: the device address it stands for is looked up once per device below and
// that pointer is what host code passes on.
static __device__ __align__(256) unsigned char scratch[RLS_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];      // per device: address of its copy of `scratch` (null until looked up)

// address of the current device's copy of the array; looked up on the first call on that device
int32_t scratch_of_current_device(void **out)
{
    int dev = -1;
    RLS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return RLS_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        RLS_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return RLS_ERR_WORKSPACE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RLS_OK;
}

}  // namespace

extern "C" int32_t rls_kmeans_sweep_static(const float *X_dev, int64_t N, int32_t d, int64_t ldx, int32_t k_min,
                                           int32_t k_max, int32_t iters, uint64_t seed, const int64_t *init_idx_dev,
                                           int32_t *labels_dev, float *centroids_dev, double *inertia_dev,
                                           double *inertia_trace_dev, int32_t *status_dev, void *stream)
{
    // sizes beyond the fixed workspace are turned down before anything is enqueued
    const int64_t need = rls_kmeans_sweep_workspace_bytes(N, d, k_min, k_max, 1);
    if (need < 0) return (int32_t)need;
    if (need > (int64_t)RLS_STATIC_WORKSPACE_BYTES) return RLS_ERR_WORKSPACE;
    void *ws = nullptr;
    const int32_t rc = scratch_of_current_device(&ws);
    if (rc != RLS_OK) return rc;
    return rls_kmeans_sweep(X_dev, N, d, ldx, k_min, k_max, iters, seed, init_idx_dev, labels_dev, centroids_dev,
                            inertia_dev, inertia_trace_dev, status_dev, ws, (int64_t)RLS_STATIC_WORKSPACE_BYTES, stream);
}
