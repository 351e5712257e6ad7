// k-means++ seeding chain (D^2 sampling) for the k-means runs of Algorithm 1 (Sec. 4.2 of the paper;
// the paper leaves the initialisation open, the chain is this library's choice).
//
// Step j keeps, per point, the fp64 squared distance D_i to the nearest of the j centres chosen so
// far, draws r = u_j * sum(D) with u_j from SplitMix64, and takes the first point whose running
// prefix of D exceeds r.  Distances use the direct form sum_l (x_l - c_l)^2 in fp64, ascending l,
// with separately rounded multiply and add.  Sums are hierarchical (thread -> wave -> block ->
// blocks) in a fixed order, so a chain is reproducible run to run.
//
// Most rows are never read after the first steps: with each point the position a_i of its nearest centre is kept, and
// when centre c is added a point with D_i <= |c_{a_i} - c|^2 / 4 cannot come closer to c than it is to c_{a_i}
// (triangle inequality: |x_i - c| >= |c_{a_i} - c| - |x_i - c_{a_i}| >= sqrt(D_i)), so D_i stays and the row is not
// fetched.  The bound carries a margin of 2^-30, far above the rounding of the fp64 sums, so every skipped point is one
// whose computed distance would not have been smaller: D, the block sums and the chain are the same with and without it.
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
// block sums are the same in every run.  A point whose D_i is at most thr[a_i] (a quarter of the squared distance of its
// nearest centre to the newest one, written by the pick kernel) keeps D_i without a look at its row.  When rows can be
// read 16 bytes at a time, the rows still wanted of 256 points at a time travel through LDS: consecutive lanes read
// consecutive 16 bytes of the row block (every cache line is fetched by one instruction), and each thread then reads its
// row back from LDS (rows of d + 4 floats: conflict free).  D_i and a_i of the next 256 points, then the rows wanted
// among them, are requested before the arithmetic on the current ones.
// Q: 16-byte units per row when rows can be read that way (d = 4 Q, aligned), 0: rows are read element by element.
struct SeedState {
    double *mind;            // fp64 [N] squared distance to the nearest centre so far
    double *bsum;            // fp64 [seed blocks] block sums of mind
    unsigned char *near;     // [N] chain position of that nearest centre
    double *thr;             // fp64 [k_max] per earlier centre: (1 - 2^-30) / 4 of its squared distance to the newest centre
    int64_t mind_bs, bsum_bs, near_bs, thr_bs;   // batch strides, in elements
};

template <int Q>
__global__ void __launch_bounds__(256) seed_update_kernel(const float *__restrict__ X, int64_t N, int d, int64_t ldx,
                                                         int64_t x_batch_stride, const int64_t *__restrict__ chain,
                                                         int64_t chain_batch_stride, int j, SeedState st)
{
    __shared__ __align__(16) float tile[Q > 0 ? 256 * (4 * Q + 4) : 4];
    __shared__ float cs[RLS_MAX_D];
    __shared__ double thr_s[RLS_MAX_K];
    __shared__ unsigned long long need_s[2][4];
    __shared__ double wsum[4];
    const int b = blockIdx.y;
    const float *Xb = X + (int64_t)b * x_batch_stride;
    double *D = st.mind + (int64_t)b * st.mind_bs;
    unsigned char *NR = st.near + (int64_t)b * st.near_bs;
    const int newest = j - 1;                        // chain position of the centre this step adds
    const int64_t centre = chain[(int64_t)b * chain_batch_stride + newest];
    if (threadIdx.x < d) cs[threadIdx.x] = Xb[centre * ldx + threadIdx.x];
    if ((int)threadIdx.x < newest) thr_s[threadIdx.x] = st.thr[(int64_t)b * st.thr_bs + threadIdx.x];
    double local = 0.0;
    const int64_t base = (int64_t)blockIdx.x * kSeedBlock;
    constexpr int kIter = kSeedBlock / 256;
    const bool first = j == 1;                       // no distances yet: every row is read
    if constexpr (Q > 0) {
        constexpr int q = Q;                         // 16-byte units per row
        constexpr int rs = 4 * Q + 4;                // row stride of the tile, in floats
        constexpr int kMaxQ = Q;
        float stage[kMaxQ][4];
        // unit u = tid + 256 e of a row block is 16 bytes of row u / q at feature 4 (u % q)
        int urow[kMaxQ], ucol[kMaxQ];
#pragma unroll
        for (int e = 0; e < kMaxQ; ++e) {
            const int u = (int)threadIdx.x + 256 * e;
            urow[e] = u / q;
            ucol[e] = 4 * (u % q);
        }
        const int wave = (int)threadIdx.x >> 6;
        double old[kIter];
        int nr[kIter];
        bool need[kIter];
        // state of this thread's point of row block I (points past the end: never wanted)
#define RLS_SEED_STATE(I)                                                                                                \
    do {                                                                                                                 \
        const int64_t p_ = base + threadIdx.x + 256 * (I);                                                               \
        old[I] = 0.0; nr[I] = 0;                                                                                         \
        if (p_ < N && !first) { old[I] = D[p_]; nr[I] = NR[p_]; }                                                        \
    } while (0)
        // which rows of block I are wanted: one bit per point, one word per wave
#define RLS_SEED_WANT(I)                                                                                                 \
    do {                                                                                                                 \
        const int64_t p_ = base + threadIdx.x + 256 * (I);                                                               \
        need[I] = p_ < N && (first || !(old[I] <= thr_s[nr[I] & (RLS_MAX_K - 1)]));                                                        \
        const unsigned long long m_ = __ballot(need[I]);                                                                 \
        if ((threadIdx.x & 63) == 0) need_s[(I) & 1][wave] = m_;                                                         \
    } while (0)
        // (written out with constant indices: the staged rows stay in registers)
#define RLS_SEED_REQUEST(I)                                                                                              \
    do {                                                                                                                 \
        const int64_t row0_ = base + 256 * (I);                                                                          \
        _Pragma("unroll") for (int e = 0; e < kMaxQ; ++e) {                                                              \
            if ((need_s[(I) & 1][urow[e] >> 6] >> (urow[e] & 63)) & 1ull) {                                              \
                const float4 v_ = *reinterpret_cast<const float4 *>(Xb + min(row0_ + urow[e], N - 1) * ldx + ucol[e]);   \
                stage[e][0] = v_.x; stage[e][1] = v_.y; stage[e][2] = v_.z; stage[e][3] = v_.w;                          \
            }                                                                                                            \
        }                                                                                                                \
    } while (0)
#pragma unroll
        for (int e = 0; e < kMaxQ; ++e) stage[e][0] = stage[e][1] = stage[e][2] = stage[e][3] = 0.0f;
        RLS_SEED_STATE(0);
        __syncthreads();                             // cs and thr_s are there
        RLS_SEED_WANT(0);
        __syncthreads();
        RLS_SEED_REQUEST(0);
        if (kIter > 1 && base + 256 < N) RLS_SEED_STATE(1);
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            if (base + 256 * i >= N) break;          // same for the whole workgroup
            __syncthreads();                         // the tile is free
#pragma unroll
            for (int e = 0; e < kMaxQ; ++e) {
                *reinterpret_cast<float4 *>(tile + urow[e] * rs + ucol[e]) = make_float4(stage[e][0], stage[e][1], stage[e][2], stage[e][3]);
            }
            const bool more = i + 1 < kIter && base + 256 * (i + 1) < N;
            if (more) RLS_SEED_WANT(i + 1 < kIter ? i + 1 : i);
            __syncthreads();                         // the tile, and which rows of the next block are wanted
            if (more) {
                RLS_SEED_REQUEST(i + 1 < kIter ? i + 1 : i);
                if (i + 2 < kIter && base + 256 * (i + 2) < N) RLS_SEED_STATE(i + 2 < kIter ? i + 2 : i);
            }
            const int64_t p = base + threadIdx.x + 256 * i;
            if (p < N) {
                double cur = old[i];
                if (need[i]) {
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
                    if (first || acc < cur) {
                        cur = acc;
                        D[p] = acc;
                        NR[p] = (unsigned char)newest;
                    }
                }
                local = __dadd_rn(local, cur);
            }
        }
#undef RLS_SEED_REQUEST
#undef RLS_SEED_WANT
#undef RLS_SEED_STATE
    } else {
        __syncthreads();
        for (int i = 0; i < kIter; ++i) {
            const int64_t p = base + threadIdx.x + 256 * i;
            if (p < N) {
                double cur = 0.0;
                bool want = true;
                if (!first) {
                    cur = D[p];
                    want = !(cur <= thr_s[NR[p] & (RLS_MAX_K - 1)]);
                }
                if (want) {
                    const float *x = Xb + p * ldx;
                    double acc = 0.0;
                    for (int l = 0; l < d; ++l) {
                        const double diff = __dsub_rn((double)x[l], (double)cs[l]);
                        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
                    }
                    if (first || acc < cur) {
                        cur = acc;
                        D[p] = acc;
                        NR[p] = (unsigned char)newest;
                    }
                }
                local = __dadd_rn(local, cur);
            }
        }
    }
    // block sum in fixed order: wave butterfly-free reduction via scan's last lane, then 4 waves in order
    const double incl = wave_inclusive_scan(local);
    if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = incl;
    __syncthreads();
    if (threadIdx.x == 0)
        st.bsum[(int64_t)b * st.bsum_bs + blockIdx.x] = __dadd_rn(__dadd_rn(wsum[0], wsum[1]), __dadd_rn(wsum[2], wsum[3]));
}

// one workgroup per space: total, draw, locate the block, locate the point; then, for the update that follows, the
// bound of every earlier centre: a quarter of its squared distance to the centre just drawn, less a margin
__global__ void __launch_bounds__(1024) seed_pick_kernel(SeedList seeds, int b0, const float *__restrict__ X, int64_t N, int d,
                                                        int64_t ldx, int64_t x_batch_stride, int j, int seed_blocks,
                                                        SeedState st, int64_t *chain, int64_t chain_batch_stride)
{
    static_assert(RLS_MAX_K * 8 <= 1024 && RLS_MAX_D <= 32, "eight threads fetch one earlier centre, four features each");
    __shared__ double wtot[16];
    __shared__ double s_prefix_before;   // prefix of all blocks before the chosen block
    __shared__ int s_block;
    __shared__ int s_pick;
    __shared__ double s_total;
    __shared__ long long s_final;
    __shared__ float crow_s[RLS_MAX_K][RLS_MAX_D + 1];   // the earlier centres
    __shared__ float cnew_s[RLS_MAX_D];
    const int b = b0 + blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double *BS = st.bsum + (int64_t)b * st.bsum_bs;
    const double *D = st.mind + (int64_t)b * st.mind_bs;
    int64_t *ch = chain + (int64_t)b * chain_batch_stride;
    const float *Xb = X + (int64_t)b * x_batch_stride;

    // rows of the centres chosen so far (positions 0 .. j-1): requested now, used at the end
    {
        const int m = tid >> 3, l0 = 4 * (tid & 7);
        if (m < j) {
            const float *row = Xb + ch[m] * ldx;
            for (int l = l0; l < l0 + 4 && l < d; ++l) crow_s[m][l] = row[l];
        }
    }

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
            s_final = pick;
        }
    } else {
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
        if (tid == 0) s_final = (long long)blk * kSeedBlock + s_pick;
    }
    __syncthreads();
    const long long pick = s_final;
    if (tid == 0) ch[j] = pick;
    // bounds for the update with this centre (a pick outside the data, which valid arguments never give: no skipping)
    const bool inside = pick >= 0 && pick < N;
    if (tid < d) cnew_s[tid] = inside ? Xb[pick * ldx + tid] : 0.0f;
    __syncthreads();
    if (tid < j) {
        double dcc = 0.0;
        for (int l = 0; l < d; ++l) {
            const double diff = (double)crow_s[tid][l] - (double)cnew_s[l];
            dcc += diff * diff;
        }
        const double bound = dcc * (0.25 * (1.0 - 0x1.0p-30));
        st.thr[(int64_t)b * st.thr_bs + tid] = inside ? bound : -1.0;
    }
}

}  // namespace

hipError_t launch_seed_chain(const float *X, int64_t N, int32_t d, int64_t ldx, int64_t x_batch_stride, int32_t batch,
                             int32_t k_max, const uint64_t *seeds_host, int64_t *chain, int64_t chain_batch_stride,
                             char *ws, const SweepLayout &L, hipStream_t s, int32_t j_begin)
{
    // positions j_begin .. k_max-1 of the chain are produced; the distance state of an earlier call for the same
    // chain (positions 0 .. j_begin-1) must still be in the workspace
    const int32_t seed_blocks = L.seed_blocks;
    for (int b0 = 0; b0 < batch; b0 += 64) {
        const int nb = batch - b0 < 64 ? batch - b0 : 64;
        SeedList sl;
        for (int i = 0; i < 64; ++i) sl.seed[i] = seeds_host[b0 + (i < nb ? i : 0)];
        char *wsb = ws + (int64_t)b0 * L.per_batch;
        SeedState st;
        st.mind = reinterpret_cast<double *>(wsb + L.mind); st.mind_bs = L.per_batch / 8;
        st.bsum = reinterpret_cast<double *>(wsb + L.bsum); st.bsum_bs = L.per_batch / 8;
        st.near = reinterpret_cast<unsigned char *>(wsb + L.near); st.near_bs = L.per_batch;
        st.thr = reinterpret_cast<double *>(wsb + L.seedthr); st.thr_bs = L.per_batch / 8;
        if (j_begin == 0) hipLaunchKernelGGL(seed_first_kernel, dim3(nb), dim3(64), 0, s, sl, b0, N, chain, chain_batch_stride);
        for (int j = j_begin > 1 ? j_begin : 1; j < k_max; ++j) {
            const float *Xg = X + (int64_t)b0 * x_batch_stride;
            // rows 16 bytes at a time when every space's rows allow it
            const bool vec = (d % 4 == 0) && (ldx % 4 == 0) && (x_batch_stride % 4 == 0 || nb == 1) &&
                             ((reinterpret_cast<uintptr_t>(Xg) & 15) == 0);
#define RLS_SEED_UPDATE(QV)                                                                                              \
    hipLaunchKernelGGL(seed_update_kernel<QV>, dim3(seed_blocks, nb), dim3(256), 0, s, Xg, N, (int)d, ldx,                \
                       x_batch_stride, chain + (int64_t)b0 * chain_batch_stride, chain_batch_stride, j, st)
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
            hipLaunchKernelGGL(seed_pick_kernel, dim3(nb), dim3(1024), 0, s, sl, 0, Xg, N, (int)d, ldx, x_batch_stride, j,
                               (int)seed_blocks, st, chain + (int64_t)b0 * chain_batch_stride, chain_batch_stride);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rls
