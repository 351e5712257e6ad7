// k-means++ seeding chain (D^2 sampling) for the k-means runs of Algorithm 1 (Sec. 4.2 of the paper;
// the paper leaves the initialisation open, the chain is this library's choice).
//
// Step j keeps, per point, the fp64 squared distance D_i to the nearest of the j centres chosen so
// far, draws r = u_j * sum(D) with u_j from SplitMix64, and takes the first point whose running
// prefix of D exceeds r.  Distances use the direct form sum_l (x_l - c_l)^2 in fp64, ascending l,
// with separately rounded multiply and add.  Sums are hierarchical (thread -> wave -> block ->
// blocks) in a fixed order, so a chain is reproducible run to run.
#include "rls_internal.h"

namespace rls {

namespace {

__device__ inline uint64_t splitmix64(uint64_t seed, uint64_t j)
{
    uint64_t z = seed + (j + 1) * 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

__device__ inline double uniform01(uint64_t seed, uint64_t j)
{
    return (double)(splitmix64(seed, j) >> 11) * 0x1.0p-53;
}

struct SeedList {
    uint64_t seed[64];
};

__global__ void seed_first_kernel(SeedList seeds, int b0, int64_t N, int64_t *chain, int64_t chain_batch_stride)
{
    const int b = b0 + blockIdx.x;
    if (threadIdx.x != 0) return;
    int64_t first = (int64_t)(uniform01(seeds.seed[blockIdx.x], 0) * (double)N);
    if (first >= N) first = N - 1;
    chain[(int64_t)b * chain_batch_stride] = first;
}

// inclusive scan / sum over a 1024-thread block in fixed order; `tmp` holds 17 doubles
__device__ inline double wave_inclusive_scan(double v)
{
    const int lane = threadIdx.x & 63;
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(v, off, 64);
        if (lane >= off) v = __dadd_rn(v, o);
    }
    return v;
}

// D_i <- min(D_i, |x_i - c|^2) for the newest centre, plus one sum per block of kSeedBlock points.
// A thread owns points base + tid + 256 i; which thread sums which point, and in which order, never changes, so the
// block sums are the same in every run.  When rows can be read 16 bytes at a time, 256 rows at a time travel through
// LDS: consecutive lanes read consecutive 16 bytes of the row block (every cache line is fetched by one instruction;
// a lane that walks its own row touches a line eight times, and with 256 lines per workgroup in flight the
// first-level cache has dropped it in between), and each thread then reads its row back from LDS (rows of d + 4
// floats: conflict free).  The rows of the next 256 points are requested before the arithmetic on the current ones.
// Q: 16-byte units per row when rows can be read that way (d = 4 Q, aligned), 0: rows are read element by element.
template <int Q>
__global__ void __launch_bounds__(256) seed_update_kernel(const float *__restrict__ X, int64_t N, int d, int64_t ldx,
                                                         int64_t x_batch_stride, const int64_t *__restrict__ chain,
                                                         int64_t chain_batch_stride, int j, double *__restrict__ mind,
                                                         int64_t mind_batch_stride, double *__restrict__ bsum,
                                                         int64_t bsum_batch_stride)
{
    __shared__ __align__(16) float tile[Q > 0 ? 256 * (4 * Q + 4) : 4];
    __shared__ float cs[RLS_MAX_D];
    __shared__ double wsum[4];
    const int b = blockIdx.y;
    const float *Xb = X + (int64_t)b * x_batch_stride;
    double *D = mind + (int64_t)b * mind_batch_stride;
    const int64_t centre = chain[(int64_t)b * chain_batch_stride + (j - 1)];
    if (threadIdx.x < d) cs[threadIdx.x] = Xb[centre * ldx + threadIdx.x];
    double local = 0.0;
    const int64_t base = (int64_t)blockIdx.x * kSeedBlock;
    constexpr int kIter = kSeedBlock / 256;
    if constexpr (Q > 0) {
        constexpr int q = Q;                         // 16-byte units per row
        constexpr int rs = 4 * Q + 4;                // row stride of the tile, in floats
        constexpr int kMaxQ = Q;
        float stage[kMaxQ][4];
        // unit u = tid + 256 e of a row block is 16 bytes of row u / q at feature 4 (u % q); rows past the end of the
        // data are clamped to the last row (read, never used)
        int urow[kMaxQ], ucol[kMaxQ];
#pragma unroll
        for (int e = 0; e < kMaxQ; ++e) {
            const int u = (int)threadIdx.x + 256 * e;
            urow[e] = u / q;
            ucol[e] = 4 * (u % q);
        }
        // (written out with constant indices: the staged rows stay in registers)
#define RLS_SEED_REQUEST(I)                                                                                              \
    do {                                                                                                                 \
        const int64_t row0_ = base + 256 * (I);                                                                          \
        _Pragma("unroll") for (int e = 0; e < kMaxQ; ++e) {                                                              \
            const float4 v_ = *reinterpret_cast<const float4 *>(Xb + min(row0_ + urow[e], N - 1) * ldx + ucol[e]);       \
            stage[e][0] = v_.x; stage[e][1] = v_.y; stage[e][2] = v_.z; stage[e][3] = v_.w;                              \
        }                                                                                                                \
    } while (0)
        RLS_SEED_REQUEST(0);
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            if (base + 256 * i >= N) break;          // same for the whole workgroup
            __syncthreads();                         // the tile is free (and, the first time, cs is there)
#pragma unroll
            for (int e = 0; e < kMaxQ; ++e) {
                *reinterpret_cast<float4 *>(tile + urow[e] * rs + ucol[e]) = make_float4(stage[e][0], stage[e][1], stage[e][2], stage[e][3]);
            }
            if (i + 1 < kIter && base + 256 * (i + 1) < N) RLS_SEED_REQUEST(i + 1);
            __syncthreads();
            const int64_t p = base + threadIdx.x + 256 * i;
            if (p < N) {
                const float *x = tile + threadIdx.x * rs;
                double acc = 0.0;
#pragma unroll
                for (int l = 0; l < 4 * Q; l += 4) {
                    const float4 xv = *reinterpret_cast<const float4 *>(x + l);
                    double diff = __dsub_rn((double)xv.x, (double)cs[l]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)xv.y, (double)cs[l + 1]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)xv.z, (double)cs[l + 2]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    diff = __dsub_rn((double)xv.w, (double)cs[l + 3]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                }
                double cur = acc;
                if (j > 1) {
                    const double old = D[p];
                    cur = acc < old ? acc : old;
                }
                D[p] = cur;
                local = __dadd_rn(local, cur);
            }
        }
#undef RLS_SEED_REQUEST
    } else {
        __syncthreads();
        for (int i = 0; i < kIter; ++i) {
            const int64_t p = base + threadIdx.x + 256 * i;
            if (p < N) {
                const float *x = Xb + p * ldx;
                double acc = 0.0;
                for (int l = 0; l < d; ++l) {
                    const double diff = __dsub_rn((double)x[l], (double)cs[l]);
                    acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                }
                double cur = acc;
                if (j > 1) {
                    const double old = D[p];
                    cur = acc < old ? acc : old;
                }
                D[p] = cur;
                local = __dadd_rn(local, cur);
            }
        }
    }
    // block sum in fixed order: wave butterfly-free reduction via scan's last lane, then 4 waves in order
    const double incl = wave_inclusive_scan(local);
    if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = incl;
    __syncthreads();
    if (threadIdx.x == 0)
        bsum[(int64_t)b * bsum_batch_stride + blockIdx.x] = __dadd_rn(__dadd_rn(wsum[0], wsum[1]), __dadd_rn(wsum[2], wsum[3]));
}

// one workgroup per space: total, draw, locate the block, locate the point
__global__ void __launch_bounds__(1024) seed_pick_kernel(SeedList seeds, int b0, int64_t N, int j, int seed_blocks,
                                                        const double *__restrict__ mind, int64_t mind_batch_stride,
                                                        const double *__restrict__ bsum, int64_t bsum_batch_stride,
                                                        int64_t *chain, int64_t chain_batch_stride)
{
    __shared__ double wtot[16];
    __shared__ double s_prefix_before;   // prefix of all blocks before the chosen block
    __shared__ int s_block;
    __shared__ int s_pick;
    __shared__ double s_total;
    const int b = b0 + blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double *BS = bsum + (int64_t)b * bsum_batch_stride;
    const double *D = mind + (int64_t)b * mind_batch_stride;
    int64_t *ch = chain + (int64_t)b * chain_batch_stride;

    // segment of blocks per thread
    const int per = (seed_blocks + 1023) / 1024;
    const int s0 = min(tid * per, seed_blocks), s1 = min(s0 + per, seed_blocks);
    double local = 0.0;
    for (int s = s0; s < s1; ++s) local = __dadd_rn(local, BS[s]);
    double incl = wave_inclusive_scan(local);
    if (lane == 63) wtot[wave] = incl;
    if (tid == 0) { s_block = 0x7fffffff; s_pick = 0x7fffffff; }
    __syncthreads();
    double wbase = 0.0;
    for (int w = 0; w < wave; ++w) wbase = __dadd_rn(wbase, wtot[w]);
    if (tid == 1023) s_total = __dadd_rn(wbase, incl);
    __syncthreads();
    const double S = s_total;
    if (!(S > 0.0)) {
        // every point coincides with a chosen centre: smallest index not chosen yet
        if (tid == 0) {
            int64_t pick = -1;
            for (int64_t i = 0; i < N && pick < 0; ++i) {
                bool taken = false;
                for (int m = 0; m < j; ++m) taken |= (ch[m] == i);
                if (!taken) pick = i;
            }
            ch[j] = pick;
        }
        return;
    }
    const double r = __dmul_rn(uniform01(seeds.seed[blockIdx.x], (uint64_t)j), S);
    // first block whose inclusive prefix exceeds r
    {
        double run = __dadd_rn(wbase, __dadd_rn(incl, -local));   // exclusive prefix of this thread's segment
        for (int s = s0; s < s1; ++s) {
            const double nxt = __dadd_rn(run, BS[s]);
            if (nxt > r && BS[s] > 0.0) { atomicMin(&s_block, s); break; }
            run = nxt;
        }
    }
    __syncthreads();
    int blk = s_block;
    const bool overflow = (blk == 0x7fffffff);   // r rounded up to S: take the last point with D > 0
    if (overflow) {
        __syncthreads();
        if (tid == 0) s_block = -1;
        __syncthreads();
        for (int s = s0; s < s1; ++s)
            if (BS[s] > 0.0) atomicMax(&s_block, s);
        __syncthreads();
        blk = s_block;
    }
    // exclusive prefix of the chosen block, recomputed in the same order by the thread that owns it
    if (blk >= s0 && blk < s1) {
        double run = __dadd_rn(wbase, __dadd_rn(incl, -local));
        for (int s = s0; s < blk; ++s) run = __dadd_rn(run, BS[s]);
        s_prefix_before = run;
    }
    __syncthreads();
    const double before = s_prefix_before;
    const int64_t p = (int64_t)blk * kSeedBlock + tid;
    const double v = p < N ? D[p] : 0.0;
    const double in_wave = wave_inclusive_scan(v);
    __syncthreads();
    if (lane == 63) wtot[wave] = in_wave;
    __syncthreads();
    double wb = before;
    for (int w = 0; w < wave; ++w) wb = __dadd_rn(wb, wtot[w]);
    const double prefix = __dadd_rn(wb, in_wave);
    if (!overflow) {
        if (v > 0.0 && prefix > r) atomicMin(&s_pick, tid);
        __syncthreads();
        if (s_pick == 0x7fffffff) {   // block-level and point-level rounding disagree: last positive point of the block
            __syncthreads();
            if (tid == 0) s_pick = -1;
            __syncthreads();
            if (v > 0.0) atomicMax(&s_pick, tid);
        }
    } else {
        __syncthreads();
        if (tid == 0) s_pick = -1;
        __syncthreads();
        if (v > 0.0) atomicMax(&s_pick, tid);
    }
    __syncthreads();
    if (tid == 0) ch[j] = (int64_t)blk * kSeedBlock + s_pick;
}

}  // namespace

hipError_t launch_seed_chain(const float *X, int64_t N, int32_t d, int64_t ldx, int64_t x_batch_stride, int32_t batch,
                             int32_t k_max, const uint64_t *seeds_host, int64_t *chain, int64_t chain_batch_stride,
                             double *mind, int64_t mind_batch_stride, double *bsum, int64_t bsum_batch_stride,
                             int32_t seed_blocks, hipStream_t s, int32_t j_begin)
{
    // positions j_begin .. k_max-1 of the chain are produced; the distance state of an earlier call for the same
    // chain (positions 0 .. j_begin-1) must still be in `mind`
    for (int b0 = 0; b0 < batch; b0 += 64) {
        const int nb = batch - b0 < 64 ? batch - b0 : 64;
        SeedList sl;
        for (int i = 0; i < 64; ++i) sl.seed[i] = seeds_host[b0 + (i < nb ? i : 0)];
        if (j_begin == 0) hipLaunchKernelGGL(seed_first_kernel, dim3(nb), dim3(64), 0, s, sl, b0, N, chain, chain_batch_stride);
        for (int j = j_begin > 1 ? j_begin : 1; j < k_max; ++j) {
            const float *Xg = X + (int64_t)b0 * x_batch_stride;
            // rows 16 bytes at a time when every space's rows allow it
            const bool vec = (d % 4 == 0) && (ldx % 4 == 0) && (x_batch_stride % 4 == 0 || nb == 1) &&
                             ((reinterpret_cast<uintptr_t>(Xg) & 15) == 0);
#define RLS_SEED_UPDATE(QV)                                                                                              \
    hipLaunchKernelGGL(seed_update_kernel<QV>, dim3(seed_blocks, nb), dim3(256), 0, s, Xg, N, (int)d, ldx,                \
                       x_batch_stride, chain + (int64_t)b0 * chain_batch_stride, chain_batch_stride, j,                   \
                       mind + (int64_t)b0 * mind_batch_stride, mind_batch_stride,                                         \
                       bsum + (int64_t)b0 * bsum_batch_stride, bsum_batch_stride)
            switch (vec ? d / 4 : 0) {
            case 1: RLS_SEED_UPDATE(1); break;
            case 2: RLS_SEED_UPDATE(2); break;
            case 3: RLS_SEED_UPDATE(3); break;
            case 4: RLS_SEED_UPDATE(4); break;
            case 5: RLS_SEED_UPDATE(5); break;
            case 6: RLS_SEED_UPDATE(6); break;
            case 7: RLS_SEED_UPDATE(7); break;
            case 8: RLS_SEED_UPDATE(8); break;
            default: RLS_SEED_UPDATE(0); break;
            }
#undef RLS_SEED_UPDATE
            hipLaunchKernelGGL(seed_pick_kernel, dim3(nb), dim3(1024), 0, s, sl, b0, N, j, (int)seed_blocks, mind,
                               mind_batch_stride, bsum, bsum_batch_stride, chain, chain_batch_stride);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rls
