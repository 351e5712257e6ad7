// Tree-ensemble scoring of a trajectory of configurations (cost-model query, Sec. 4.1 of the paper).
//
// One configuration per lane.  A workgroup keeps a tile of P configurations in LDS, feature-major
// (xs[f][p]): the walk reads xs[feat][lane], whose bank is lane % 32 whatever `feat` is, so these
// gathers never conflict.  The forest is streamed through LDS in chunks of whole trees with each
// internal node packed as (LDS byte offset of the feature's row, threshold bits); every lane adds the leaf
// values to its own fp32 running sum in tree order, which makes the result independent of the launch shape.
// A step of the walk is two dependent LDS reads and four vector instructions: the walk keeps the node's LDS
// address a (node n of a tree at byte b sits at b + 8 n) and moves to child 2n + 1 + c by a <- 2 a + (8 + 8 c - b).
#include <algorithm>
#include <mutex>

#include "rls_internal.h"

namespace rls {

namespace {

constexpr int kForestChunkBytes = 96 * 1024;   // with the 64 KB tile of configurations this fills the 160 KB of LDS
// Entries (internal nodes, and leaves) a thread carries in registers for the next chunk: enough for a chunk of
// kForestChunkBytes of deep trees at 512 threads.  Shallow trees have more leaves per byte (2^D leaves in 12 2^D - 8
// bytes), so the launcher also caps the trees per chunk by kStage * threads leaves.
constexpr int kStage = (kForestChunkBytes / 12 + 511) / 512 + 1;

// LDS is addressed by 32-bit byte addresses that the walk computes itself (the start of the dynamic block is folded into
// them once: as a pointer offset it is a link-time constant and would cost an addition per read)
typedef __attribute__((address_space(3))) unsigned char lds_byte;
__device__ inline unsigned lds_address(const void *p) { return (unsigned)(uintptr_t)(lds_byte *)p; }
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
__device__ inline uint2v lds_read_u2(unsigned a) { return *(const __attribute__((address_space(3))) uint2v *)(uintptr_t)a; }
__device__ inline float lds_read_f(unsigned a) { return *(const __attribute__((address_space(3))) float *)(uintptr_t)a; }

__global__ void gbt_score_kernel(ForestArgs f, const float *__restrict__ X, int64_t N, int d, int64_t ldx,
                                 float *__restrict__ score, int trees_per_chunk)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int P = blockDim.x;
    const int n_int = (1 << f.depth) - 1;
    const int n_leaf = 1 << f.depth;
    float *xs = reinterpret_cast<float *>(smem);                                // [d][P]
    uint2 *nodes = reinterpret_cast<uint2 *>(xs + (size_t)d * P);               // [trees_per_chunk][n_int]
    float *leaves = reinterpret_cast<float *>(nodes + (size_t)trees_per_chunk * n_int);   // [trees_per_chunk][n_leaf]

    const int tid = threadIdx.x;
    const unsigned lds0 = lds_address(smem);
    const int64_t row = (int64_t)blockIdx.x * P + tid;
    const bool valid = row < N;
    {
        const float *x = X + (valid ? row : 0) * ldx;
        if (valid && (d % 4 == 0) && (ldx % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15) == 0)) {
            const float4 *x4 = reinterpret_cast<const float4 *>(x);
            for (int c = 0; c < d / 4; ++c) {
                const float4 v = x4[c];
                xs[(4 * c + 0) * P + tid] = v.x;
                xs[(4 * c + 1) * P + tid] = v.y;
                xs[(4 * c + 2) * P + tid] = v.z;
                xs[(4 * c + 3) * P + tid] = v.w;
            }
        } else {
            for (int c = 0; c < d; ++c) xs[c * P + tid] = valid ? x[c] : 0.0f;
        }
    }

    // The next chunk of the forest travels in registers while the current one is walked: its loads are issued
    // before the walk (unconditional, indices clamped) and written to LDS after it.
    int st_feat[kStage];
    float st_thr[kStage], st_leaf[kStage];
    auto fetch_chunk = [&](int t0, int tc) {
        const int n_nodes = tc * n_int, n_leaves = tc * n_leaf;
#pragma unroll
        for (int i = 0; i < kStage; ++i) {
            const int e = tid + i * P;
            const size_t en = (size_t)t0 * n_int + min(e, n_nodes - 1), el = (size_t)t0 * n_leaf + min(e, n_leaves - 1);
            st_feat[i] = f.feat[en];
            st_thr[i] = f.thr[en];
            st_leaf[i] = f.leaf[el];
        }
    };
    auto store_chunk = [&](int tc) {
        const int n_nodes = tc * n_int, n_leaves = tc * n_leaf;
#pragma unroll
        for (int i = 0; i < kStage; ++i) {
            const int e = tid + i * P;
            if (e < n_nodes) {
                const int ft = min(max(st_feat[i], 0), d - 1);
                nodes[e] = make_uint2(lds0 + (unsigned)ft * (unsigned)P * 4u, __float_as_uint(st_thr[i]));
            }
            if (e < n_leaves) leaves[e] = st_leaf[i];
        }
    };

    float sum = f.base;
    fetch_chunk(0, min(trees_per_chunk, f.n_trees));
    store_chunk(min(trees_per_chunk, f.n_trees));
    __syncthreads();   // first chunk and xs in place
    for (int t0 = 0; t0 < f.n_trees; t0 += trees_per_chunk) {
        const int tc = min(trees_per_chunk, f.n_trees - t0);
        const int tc_cap = trees_per_chunk;
        const int t_next = t0 + trees_per_chunk;
        const int tc_next = min(trees_per_chunk, f.n_trees - t_next);
        if (tc_next > 0) fetch_chunk(t_next, tc_next);
        // Four trees are walked side by side: a walk is a chain of dependent LDS reads (node, then feature value),
        // and independent chains keep more of them in flight.  The leaves are still added in tree order.
        constexpr int W = 4;
        const unsigned nodes_at = lds0 + (unsigned)((size_t)d * P * 4);        // LDS address of the node block
        const unsigned leaves_at = nodes_at + (unsigned)tc_cap * (unsigned)n_int * 8u;
        const unsigned tid4 = (unsigned)tid * 4u;
        for (int t = 0; t < tc; t += W) {
            unsigned base[W], a[W], k_left[W], k_right[W];
#pragma unroll
            for (int w = 0; w < W; ++w) {
                base[w] = nodes_at + (unsigned)min(t + w, tc - 1) * (unsigned)n_int * 8u;
                a[w] = base[w];
                k_left[w] = 8u - base[w];      // x < threshold: child 2n + 1
                k_right[w] = 16u - base[w];    // otherwise: child 2n + 2
                asm volatile("" : "+v"(k_left[w]), "+v"(k_right[w]));   // keep both as they are: one select per step
            }
            for (int lev = 0; lev < f.depth; ++lev) {
                uint2v nd[W];
#pragma unroll
                for (int w = 0; w < W; ++w) nd[w] = lds_read_u2(a[w]);
                float xv[W];
#pragma unroll
                for (int w = 0; w < W; ++w) xv[w] = lds_read_f(nd[w].x + tid4);
#pragma unroll
                for (int w = 0; w < W; ++w) a[w] = 2u * a[w] + ((xv[w] < __uint_as_float(nd[w].y)) ? k_left[w] : k_right[w]);
            }
            // leaf l of tree t + w: the walk ends at a = base + 8 (n_int + l), the leaf sits at leaves_at + 4 ((t + w) n_leaf + l)
            // = a / 2 + (leaves_at + 4 (t + w) n_leaf - 4 n_int - base / 2): one shift and one add of a scalar
#pragma unroll
            for (int w = 0; w < W; ++w)
                if (t + w < tc) sum = sum + lds_read_f((a[w] >> 1) + (leaves_at + 4u * (unsigned)((t + w) * n_leaf - n_int) - (base[w] >> 1)));
        }
        __syncthreads();   // every wave is done with this chunk
        if (tc_next > 0) store_chunk(tc_next);
        __syncthreads();
    }
    if (valid) score[row] = sum;
}

}  // namespace

hipError_t launch_gbt_score(const ForestArgs *forests_host, int32_t batch, const float *X, int64_t N, int32_t d,
                            int64_t ldx, int64_t x_batch_stride, float *score, hipStream_t s)
{
    const int P = d <= 16 ? 1024 : 512;
    static std::once_flag attr_once;
    static hipError_t attr_status = hipSuccess;
    std::call_once(attr_once, [] {
        attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(gbt_score_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (attr_status != hipSuccess) return attr_status;
    for (int32_t b = 0; b < batch; ++b) {
        const ForestArgs &f = forests_host[b];
        const int64_t tree_bytes = (((int64_t)1 << f.depth) - 1) * 8 + ((int64_t)1 << f.depth) * 4;
        // the forest chunk takes what the tile of configurations leaves of the 160 KB, at most kForestChunkBytes
        const int64_t chunk_bytes = std::min<int64_t>(kForestChunkBytes, 160 * 1024 - (int64_t)d * P * 4);
        int tpc = (int)(chunk_bytes / tree_bytes);
        // a thread stages kStage entries of the next chunk: its leaves (the larger of the two arrays) must fit
        const int64_t stage_cap = ((int64_t)kStage * P) >> f.depth;
        if (tpc > stage_cap) tpc = (int)stage_cap;
        if (tpc < 1) tpc = 1;
        if (tpc > f.n_trees) tpc = f.n_trees;
        if (((int64_t)tpc << f.depth) > (int64_t)kStage * P) return hipErrorInvalidValue;   // depth <= 12: cannot happen
        const size_t lds = (size_t)d * P * 4 + (size_t)tpc * tree_bytes;
        const unsigned grid = (unsigned)((N + P - 1) / P);
        hipLaunchKernelGGL(gbt_score_kernel, dim3(grid), dim3(P), lds, s, f, X + (int64_t)b * x_batch_stride, N, (int)d,
                           ldx, score + (int64_t)b * N, tpc);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rls
