// Tree-ensemble scoring of a trajectory of configurations (cost-model query, Sec. 4.1 of the paper).
//
// One configuration per lane.  A workgroup keeps a tile of P configurations in LDS, feature-major
// (xs[f][p]): the walk reads xs[feat][lane], whose bank is lane % 32 whatever `feat` is, so these
// gathers never conflict.  The forest is streamed through LDS in chunks of whole trees with each
// internal node packed as (LDS byte offset of the feature's row, threshold bits); every lane adds the leaf
// values to its own fp32 running sum in tree order, which makes the result independent of the launch shape.
// Every workgroup streams the whole forest, so the tile is as large as LDS allows beside a chunk of four trees
// (up to 1024 configurations), and a chunk is moved 16 bytes per lane at a time where the alignment allows.
// A step of the walk is two dependent LDS reads and four vector instructions: the walk keeps the node's LDS
// address a (node n of a tree at byte b sits at b + 8 n) and moves to child 2n + 1 + c by a <- 2 a + (8 + 8 c - b).
#include <algorithm>
#include <mutex>

#include "rls_internal.h"

namespace rls {

namespace {

constexpr int kForestChunkBytes = 96 * 1024;   // with the 64 KB tile of configurations this fills the 160 KB of LDS
constexpr int kSideBySide = 4;                 // trees a lane walks at the same time (fewer where a chunk holds fewer)
// Groups of four entries (internal nodes, and leaves) a thread carries in registers for the next chunk: enough for a
// chunk of `bytes` of deep trees.  Shallow trees have more leaves per byte (2^D leaves in 12 2^D - 8 bytes), so the
// launcher also caps the trees per chunk by 4 * groups * threads leaves.
constexpr int stage_groups(int bytes, int threads) { return (bytes / 12 + 4 * threads - 1) / (4 * threads); }

// LDS is addressed by 32-bit byte addresses that the walk computes itself (the start of the dynamic block is folded into
// them once: as a pointer offset it is a link-time constant and would cost an addition per read)
typedef __attribute__((address_space(3))) unsigned char lds_byte;
__device__ inline unsigned lds_address(const void *p) { return (unsigned)(uintptr_t)(lds_byte *)p; }
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
__device__ inline uint2v lds_read_u2(unsigned a) { return *(const __attribute__((address_space(3))) uint2v *)(uintptr_t)a; }
__device__ inline float lds_read_f(unsigned a) { return *(const __attribute__((address_space(3))) float *)(uintptr_t)a; }
__device__ inline void lds_write_u2(unsigned a, uint2v v) { *(__attribute__((address_space(3))) uint2v *)(uintptr_t)a = v; }
__device__ inline void lds_write_u4(unsigned a, uint4v v) { *(__attribute__((address_space(3))) uint4v *)(uintptr_t)a = v; }
__device__ inline void lds_write_f(unsigned a, float v) { *(__attribute__((address_space(3))) float *)(uintptr_t)a = v; }
__device__ inline void lds_write_f4(unsigned a, float4v v) { *(__attribute__((address_space(3))) float4v *)(uintptr_t)a = v; }

// P threads (= configurations of the tile), G groups of staged entries per thread, W trees walked side by side.
// `quads`: the forest's arrays start at multiples of 16 bytes and the chunks at multiples of four trees, so that a chunk
// of a multiple of four trees is moved four entries at a time.
template <int P, int G, int W>
__global__ void __launch_bounds__(P) gbt_score_kernel(ForestArgs f, const float *__restrict__ X, int64_t N, int d, int64_t ldx,
                                                      float *__restrict__ score, int trees_per_chunk, int quads)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int n_int = (1 << f.depth) - 1;
    const int n_leaf = 1 << f.depth;
    float *xs = reinterpret_cast<float *>(smem);                                // [d][P]
    // the chunk buffer behind it: [trees_per_chunk][n_int] nodes, then [trees_per_chunk][n_leaf] leaves
    const unsigned xs_bytes = (unsigned)d * (unsigned)P * 4u;
    const unsigned node_bytes = (unsigned)trees_per_chunk * (unsigned)n_int * 8u;

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
    // before the walk (unconditional, offsets clamped to the chunk) and written to LDS after it.  Every offset is a
    // 32-bit byte offset from the chunk's start in its array; staging costs a few instructions per entry, and a deep
    // tree has as many entries as a tenth of the node visits a tile pays for it.
    constexpr int E = 4 * G;
    int st_feat[E];
    float st_thr[E], st_leaf[E];
    auto fetch_chunk = [&](int t0, int tc) {
        const unsigned n_nodes = (unsigned)(tc * n_int), n_leaves = (unsigned)(tc * n_leaf);
        const char *const fc = reinterpret_cast<const char *>(f.feat + (size_t)t0 * n_int);
        const char *const hc = reinterpret_cast<const char *>(f.thr + (size_t)t0 * n_int);
        const char *const lc = reinterpret_cast<const char *>(f.leaf + (size_t)t0 * n_leaf);
        if (quads && (tc & 3) == 0) {
            const unsigned last_n = n_nodes * 4u - 16u, last_l = n_leaves * 4u - 16u;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const unsigned o = (unsigned)(tid + i * P) * 16u;
                const unsigned on = min(o, last_n), ol = min(o, last_l);
                const int4 a = *reinterpret_cast<const int4 *>(fc + on);
                const float4 h = *reinterpret_cast<const float4 *>(hc + on);
                const float4 l = *reinterpret_cast<const float4 *>(lc + ol);
                st_feat[4 * i + 0] = a.x; st_feat[4 * i + 1] = a.y; st_feat[4 * i + 2] = a.z; st_feat[4 * i + 3] = a.w;
                st_thr[4 * i + 0] = h.x; st_thr[4 * i + 1] = h.y; st_thr[4 * i + 2] = h.z; st_thr[4 * i + 3] = h.w;
                st_leaf[4 * i + 0] = l.x; st_leaf[4 * i + 1] = l.y; st_leaf[4 * i + 2] = l.z; st_leaf[4 * i + 3] = l.w;
            }
        } else {
            const unsigned last_n = n_nodes * 4u - 4u, last_l = n_leaves * 4u - 4u;
#pragma unroll
            for (int i = 0; i < E; ++i) {
                const unsigned o = (unsigned)(tid + i * P) * 4u;
                const unsigned on = min(o, last_n), ol = min(o, last_l);
                st_feat[i] = *reinterpret_cast<const int *>(fc + on);
                st_thr[i] = *reinterpret_cast<const float *>(hc + on);
                st_leaf[i] = *reinterpret_cast<const float *>(lc + ol);
            }
        }
    };
    // a node in LDS: (LDS address of its feature's row of the tile, threshold bits)
    auto row_of = [&](int ft) { return lds0 + (unsigned)min(max(ft, 0), d - 1) * (unsigned)(P * 4); };
    auto store_chunk = [&](int tc) {
        const unsigned nodes_end = (unsigned)(tc * n_int) * 8u, leaves_end = (unsigned)(tc * n_leaf) * 4u;
        const unsigned nodes_at = lds0 + xs_bytes, leaves_at = nodes_at + node_bytes;
        if (quads && (tc & 3) == 0) {
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const unsigned g = (unsigned)(tid + i * P);
                if (g * 32u < nodes_end) {
                    uint4v lo, hi;
                    lo.x = row_of(st_feat[4 * i + 0]); lo.y = __float_as_uint(st_thr[4 * i + 0]);
                    lo.z = row_of(st_feat[4 * i + 1]); lo.w = __float_as_uint(st_thr[4 * i + 1]);
                    hi.x = row_of(st_feat[4 * i + 2]); hi.y = __float_as_uint(st_thr[4 * i + 2]);
                    hi.z = row_of(st_feat[4 * i + 3]); hi.w = __float_as_uint(st_thr[4 * i + 3]);
                    lds_write_u4(nodes_at + g * 32u, lo);
                    lds_write_u4(nodes_at + g * 32u + 16u, hi);
                }
                if (g * 16u < leaves_end) {
                    float4v l;
                    l.x = st_leaf[4 * i + 0]; l.y = st_leaf[4 * i + 1]; l.z = st_leaf[4 * i + 2]; l.w = st_leaf[4 * i + 3];
                    lds_write_f4(leaves_at + g * 16u, l);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < E; ++i) {
                const unsigned e = (unsigned)(tid + i * P);
                if (e * 8u < nodes_end) {
                    uint2v n;
                    n.x = row_of(st_feat[i]); n.y = __float_as_uint(st_thr[i]);
                    lds_write_u2(nodes_at + e * 8u, n);
                }
                if (e * 4u < leaves_end) lds_write_f(leaves_at + e * 4u, st_leaf[i]);
            }
        }
    };

    float sum = f.base;
    // W trees are walked side by side: a walk is a chain of dependent LDS reads (node, then feature value),
    // and independent chains keep more of them in flight.  The leaves are still added in tree order.
    auto walk_chunk = [&](int tc) {
        const unsigned nodes_at = lds0 + xs_bytes;                             // LDS address of the node block
        const unsigned leaves_at = nodes_at + node_bytes;
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
    };
    const int tpc = trees_per_chunk;
    fetch_chunk(0, min(tpc, f.n_trees));
    store_chunk(min(tpc, f.n_trees));
    __syncthreads();   // first chunk and xs in place
    for (int t0 = 0; t0 < f.n_trees; t0 += tpc) {
        const int tc = min(tpc, f.n_trees - t0);
        const int tc_next = min(tpc, f.n_trees - (t0 + tpc));
        if (tc_next > 0) fetch_chunk(t0 + tpc, tc_next);
        walk_chunk(tc);
        __syncthreads();   // every wave is done with this chunk
        if (tc_next > 0) store_chunk(tc_next);
        __syncthreads();
    }
    if (valid) score[row] = sum;
}

using Kernel = void (*)(ForestArgs, const float *, int64_t, int, int64_t, float *, int, int);

// the kernels of one tile size: 4, 2, 1 trees side by side
struct TileKernels {
    int threads, groups;
    Kernel kernel[3];
};
constexpr int kTileSizes = 2;
static_assert(RLS_MAX_D * 896 * 4 + ((1 << RLS_MAX_DEPTH) - 1) * 8 + (1 << RLS_MAX_DEPTH) * 4 <= 160 * 1024,
              "the deepest tree fits beside the smaller tile at the largest number of features");
template <int P>
TileKernels tile_kernels()
{
    constexpr int G = stage_groups(kForestChunkBytes, P);
    return TileKernels{P, G, {gbt_score_kernel<P, G, 4>, gbt_score_kernel<P, G, 2>, gbt_score_kernel<P, G, 1>}};
}

}  // namespace

hipError_t launch_gbt_score(const ForestArgs *forests_host, int32_t batch, const float *X, int64_t N, int32_t d,
                            int64_t ldx, int64_t x_batch_stride, float *score, hipStream_t s)
{
    // tiles, largest first: with up to 32 features and trees of depth up to 12 no smaller one ever holds more trees
    static const TileKernels tiles[kTileSizes] = {tile_kernels<1024>(), tile_kernels<896>()};
    static std::once_flag attr_once;
    static hipError_t attr_status = hipSuccess;
    std::call_once(attr_once, [] {
        for (const TileKernels &t : tiles)
            for (const Kernel k : t.kernel)
                if (attr_status == hipSuccess)
                    attr_status = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (attr_status != hipSuccess) return attr_status;
    for (int32_t b = 0; b < batch; ++b) {
        const ForestArgs &f = forests_host[b];
        const int64_t tree_bytes = (((int64_t)1 << f.depth) - 1) * 8 + ((int64_t)1 << f.depth) * 4;
        // The forest chunks take what the tile of configurations leaves of the 160 KB, at most kForestChunkBytes.  Every
        // workgroup streams the whole forest, so the tile is the largest whose remainder still holds the trees a lane
        // walks side by side (failing that, the largest among those that hold the most).
        const TileKernels *tile = nullptr;
        int64_t chunk_bytes = 0;
        int best_side = 0;
        for (const TileKernels &t : tiles) {
            const int64_t space = std::min<int64_t>(kForestChunkBytes, 160 * 1024 - (int64_t)d * t.threads * 4);
            const int64_t fit = space > 0 ? space / tree_bytes : 0;
            const int side = fit >= kSideBySide ? kSideBySide : (fit >= 2 ? 2 : (fit >= 1 ? 1 : 0));
            if (side > best_side) { best_side = side; tile = &t; chunk_bytes = space; }
        }
        if (tile == nullptr) return hipErrorInvalidValue;          // one tree does not fit beside any tile
        const int P = tile->threads;
        const int groups = tile->groups;
        int tpc = (int)(chunk_bytes / tree_bytes);
        // a thread stages 4 * groups entries of the next chunk: its leaves (the larger of the two arrays) must fit
        const int64_t stage_cap = ((int64_t)4 * groups * P) >> f.depth;
        if (tpc > stage_cap) tpc = (int)stage_cap;
        if (tpc < 1) return hipErrorInvalidValue;                  // depth <= 12: cannot happen
        const int side = tpc >= 4 ? 4 : (tpc >= 2 ? 2 : 1);
        tpc -= tpc % side;
        if (tpc > f.n_trees) tpc = f.n_trees;
        const size_t lds = (size_t)d * P * 4 + (size_t)tpc * tree_bytes;
        if (lds > 160 * 1024) return hipErrorInvalidValue;
        // four entries at a time: every chunk starts at a multiple of four trees, the arrays at multiples of 16 bytes
        const int quads = (tpc % 4 == 0 || tpc == f.n_trees) &&
                          ((reinterpret_cast<uintptr_t>(f.feat) | reinterpret_cast<uintptr_t>(f.thr) |
                            reinterpret_cast<uintptr_t>(f.leaf)) & 15) == 0;
        const unsigned grid = (unsigned)((N + P - 1) / P);
        const Kernel kernel = tile->kernel[side == 4 ? 0 : (side == 2 ? 1 : 2)];
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(P), lds, s, f, X + (int64_t)b * x_batch_stride, N, (int)d, ldx,
                           score + (int64_t)b * N, tpc, quads);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rls
