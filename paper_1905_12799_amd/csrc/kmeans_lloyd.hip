// Lloyd's k-means for every k of a range at once: the "k-means(s_Theta, k)" call inside the loop of
// Algorithm 1 (Sec. 4.2 of the paper), all k side by side, iterations in lock step.
//
// Per iteration one launch of lloyd_step_kernel does, for every (group of runs, chunk of points):
//   phase 0  load a tile of points (raw fp32 into LDS, fixed-point copies into registers)
//   phase A  distances by fp32 MFMA in the expansion |c'|^2 + |x'|^2 - 2 x'.c' on data centred by the
//            column means; per point and run, the best and second-best packed (value, index) keys
//   phase B  points whose two best keys are closer than the error bound of phase A are decided
//            again in fp64 with the direct form sum_l (x_l - c_l)^2 - the arithmetic that defines
//            the assignment - so labels do not depend on fp32 cancellation
//   phase C  exact centroid sums: every member adds its fixed-point row to its cluster's int64
//            accumulators in LDS (integer adds commute, so the result is independent of order);
//            per-chunk partials go to global memory and lloyd_centroids_kernel reduces them in 128 bits,
//            rounds once to fp64, divides by the count and rounds to fp32
// The final pass replaces phase C by the fp64 loss of every point and the label output.
#include "rls_internal.h"

namespace rls {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;
constexpr float kPadNorm = 1.0e30f;           // squared norm given to padding rows: never the minimum
constexpr int kBigKey = 0x7f000000;           // larger than any key of a finite distance below 1.7e38

__host__ __device__ constexpr int tile_points_of(int dp) { return dp == 32 ? 128 : 256; }

// ---- LDS carve of lloyd_step_kernel (bytes), shared by the planner and the kernel ------------
struct Carve {
    int xs, opA, cn, sums, cnts, labels, queue, misc, total;
};
__host__ __device__ inline Carve carve_lds(int dp, int n_tiles, int real_rows)
{
    const int tp = tile_points_of(dp);
    Carve c;
    int off = 0;
    c.xs = off;      off += tp * (dp + 4) * 4;
    c.opA = off;     off += n_tiles * 32 * dp * 4;
    c.cn = off;      off += n_tiles * 32 * 4;
    c.sums = off;    off += real_rows * (dp + 1) * 8;
    c.cnts = off;    off += (real_rows * 4 + 15) / 16 * 16;
    c.labels = off;  off += tp * 8;
    c.queue = off;   off += tp * 8 * 2;
    c.misc = off;    off += 1024;
    c.total = off;
    return c;
}

struct StepArgs {
    const float *X;
    int64_t N;
    int32_t d;
    int64_t ldx;
    int64_t x_bs;            // elements between spaces of a batch
    const float *C;          // current centroids, packed [total_rows][d]
    int64_t c_bs;
    int32_t *labels;         // [n_runs][N] or null (final pass only)
    int64_t lab_bs;
    const int32_t *status;   // [batch]
    char *ws;                // workspace base
    int64_t ws_bs;           // bytes per batch element
    int64_t off_colinfo, off_opA, off_cn, off_cnmax, off_psum, off_pcnt, off_pj, off_losum;
};

__device__ inline int med3_i32(int a, int b, int c)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// x * 2^shift as an integer; exact whenever x is a multiple of 2^-shift
__device__ inline long long to_fixed(float x, int shift)
{
    const unsigned u = __float_as_uint(x);
    int e = (int)((u >> 23) & 0xffu);
    unsigned m = u & 0x7fffffu;
    if (e == 0) {
        if (m == 0) return 0;
        e = 1;
    } else {
        m |= 0x800000u;
    }
    const int sh = e - 150 + shift;
    long long q;
    if (sh >= 0) q = (long long)m << (sh > 39 ? 39 : sh);
    else q = (long long)(m >> (-sh > 31 ? 31 : -sh));
    return (u >> 31) ? -q : q;
}

// The part of x below the column grid 2^-shift, scaled by 2^(shift + kLowBits): the bits that to_fixed drops.
// Non-zero only in columns whose values span more than kGridBits binary digits.
constexpr int kGridBits = 44;   // bits of |x * 2^shift| kept by the main accumulator
constexpr int kLowBits = 36;    // further bits kept by the low accumulator
__device__ inline long long fixed_low(float x, int shift)
{
    const unsigned u = __float_as_uint(x);
    int e = (int)((u >> 23) & 0xffu);
    unsigned m = u & 0x7fffffu;
    if (e == 0) {
        if (m == 0) return 0;
        e = 1;
    } else {
        m |= 0x800000u;
    }
    const int sh = e - 150 + shift;
    if (sh >= 0) return 0;
    const int drop = -sh > 24 ? 24 : -sh;                     // dropped bits of the 24-bit significand
    const unsigned long long low = (unsigned long long)(m & ((1u << drop) - 1u));
    // value of the dropped bits is low * 2^sh on the grid scale; on the low scale it is low * 2^(sh + kLowBits)
    const int up = sh + kLowBits;
    const long long q = up >= 0 ? (long long)(low << up) : (long long)(low >> (-up > 63 ? 63 : -up));
    return (u >> 31) ? -q : q;
}

__device__ inline double sqdist64(const float *x, const float *c, int d)
{
    double acc = 0.0;
    for (int l = 0; l < d; ++l) {
        const double diff = __dsub_rn((double)x[l], (double)c[l]);
        acc = __dadd_rn(acc, __dmul_rn(diff, diff));
    }
    return acc;
}

// The index that phase A packs into the low 7 bits of a key is the centroid index within the run:
// centroid j lives in tile (j/4)/S, slot (j/4)%S of its run, row j%4 (see GroupDesc).
template <int S>
__device__ inline int key_index(int t, int a, int i)
{
    if (S == 1) return 4 * t + i;
    if (S == 2) return 8 * t + 4 * (a & 1) + i;
    if (S == 4) return 16 * t + 4 * a + i;
    return 32 * t + 4 * a + i;   // S == 8: bit 4 (the half-wave) is added after the tile loop
}
template <int S>
__device__ inline int state_of(int a) { return S == 1 ? a : (S == 2 ? (a >> 1) : 0); }

// Phase A for one wave: NB blocks of 32 points against all tiles of the group.
template <int DP, int S>
__device__ inline void phase_a(const float *xs, const float *opA_s, const float *cn_s, const float *mu_s,
                               const float *cnmax_s, unsigned char *labels_s, unsigned short *queue, int *qcount,
                               int n_tiles, int n_runs_g, int nvalid, float eps_a)
{
    constexpr int TP = tile_points_of(DP);
    constexpr int NB = TP / 128;
    constexpr int H = DP / 2;                       // features per half-wave
    constexpr int ST = S == 1 ? 4 : (S == 2 ? 2 : 1);
    constexpr int XS = DP + 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hl = lane >> 5;

    float mu[H];
#pragma unroll
    for (int s = 0; s < H; ++s) mu[s] = mu_s[hl * H + s];

    float b[NB][H];
    float xn[NB];
    int m1[NB][ST], m2[NB][ST];
#pragma unroll
    for (int pb = 0; pb < NB; ++pb) {
        const int p = wave * 32 * NB + pb * 32 + n;
        const float4 *row = reinterpret_cast<const float4 *>(xs + p * XS + hl * H);
        float part = 0.0f;
#pragma unroll
        for (int c4 = 0; c4 < H / 4; ++c4) {
            const float4 v = row[c4];
            b[pb][4 * c4 + 0] = v.x - mu[4 * c4 + 0];
            b[pb][4 * c4 + 1] = v.y - mu[4 * c4 + 1];
            b[pb][4 * c4 + 2] = v.z - mu[4 * c4 + 2];
            b[pb][4 * c4 + 3] = v.w - mu[4 * c4 + 3];
        }
#pragma unroll
        for (int s = 0; s < H; ++s) part = fmaf(b[pb][s], b[pb][s], part);
        xn[pb] = part + __shfl_xor(part, 32, 64);
#pragma unroll
        for (int st = 0; st < ST; ++st) { m1[pb][st] = kBigKey; m2[pb][st] = kBigKey; }
    }

    for (int t = 0; t < n_tiles; ++t) {
        float a[H];
#pragma unroll
        for (int c4 = 0; c4 < H / 4; ++c4) {
            const float4 v = *reinterpret_cast<const float4 *>(opA_s + ((((t * 2 + hl) * (H / 4) + c4) * 32 + n) << 2));
            a[4 * c4 + 0] = v.x; a[4 * c4 + 1] = v.y; a[4 * c4 + 2] = v.z; a[4 * c4 + 3] = v.w;
        }
        floatx16 cnv;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(cn_s + t * 32 + 8 * q + 4 * hl);
            cnv[4 * q + 0] = v.x; cnv[4 * q + 1] = v.y; cnv[4 * q + 2] = v.z; cnv[4 * q + 3] = v.w;
        }
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            floatx16 acc = cnv;
#pragma unroll
            for (int s = 0; s < H; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[pb][s], acc, 0, 0, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = acc[4 * q + i] + xn[pb];
                    const int key = (__float_as_int(v) & (int)0xffffff80) | key_index<S>(t, q, i);
                    const int st = state_of<S>(q);
                    m2[pb][st] = med3_i32(m1[pb][st], m2[pb][st], key);
                    m1[pb][st] = min(m1[pb][st], key);
                }
            }
        }
    }

#pragma unroll
    for (int pb = 0; pb < NB; ++pb) {
        const int p = wave * 32 * NB + pb * 32 + n;
        if (S == 8) {
            // the run spans both half-waves: add the half bit to the index, then merge with the partner lane
            int k1 = m1[pb][0], k2 = m2[pb][0];
            if (k1 != kBigKey) k1 |= hl << 4;
            if (k2 != kBigKey) k2 |= hl << 4;
            const int o1 = __shfl_xor(k1, 32, 64), o2 = __shfl_xor(k2, 32, 64);
            m1[pb][0] = min(k1, o1);
            m2[pb][0] = min(max(k1, o1), min(k2, o2));
        }
#pragma unroll
        for (int st = 0; st < ST; ++st) {
            const int rl = S == 8 ? 0 : hl * ST + st;     // run within the group
            const bool writer = (S == 8) ? (hl == 0) : true;
            if (!writer || rl >= n_runs_g) continue;
            unsigned char lab = 0xff;
            if (p < nvalid) {
                const int k1 = m1[pb][st], k2 = m2[pb][st];
                lab = (unsigned char)(k1 & 127);
                const float f1 = __int_as_float(k1 & (int)0xffffff80), f2 = __int_as_float(k2 & (int)0xffffff80);
                // error bound of the fp32 expansion (rounding of norms, products and the centring) plus the
                // 7 mantissa bits given up to the index in each key
                const float tol = eps_a * (xn[pb] + cnmax_s[rl]) + 6.2e-5f * fabsf(f2) + 1.0e-30f;
                if (!(f2 - f1 > tol)) {
                    const int slot = atomicAdd(qcount, 1);
                    queue[slot] = (unsigned short)(p | (rl << 8));
                }
            }
            labels_s[p * 8 + rl] = lab;
        }
    }
}

template <int DP, bool FINAL, bool TRACE>
__global__ void __launch_bounds__(kThreads) lloyd_step_kernel(SweepPlan plan, StepArgs a)
{
    constexpr int TP = tile_points_of(DP);
    constexpr int XS = DP + 4;
    constexpr int PPP = kThreads / DP;            // points per pass of the (point, feature) mapping
    constexpr int NQ = TP / PPP;                  // passes per tile
    constexpr bool LOSS = FINAL || TRACE;
    extern __shared__ __align__(16) unsigned char smem[];

    const int b = blockIdx.y;
    if (a.status[b] != 0) return;
    const int gi = blockIdx.x % plan.n_groups;
    const int chunk = blockIdx.x / plan.n_groups;
    const GroupDesc g = plan.g[gi];
    const int d = a.d;
    const int k0 = plan.k_min + g.run0;                                   // k of the group's first run
    const int grow0 = rows_before(plan.k_min, g.run0);                    // first centroid row of the group
    const int real_rows = rows_before(plan.k_min, g.run0 + g.n_runs) - grow0;
    const Carve cv = carve_lds(DP, g.n_tiles, real_rows);

    float *xs = reinterpret_cast<float *>(smem + cv.xs);
    float *opA_s = reinterpret_cast<float *>(smem + cv.opA);
    float *cn_s = reinterpret_cast<float *>(smem + cv.cn);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(smem + cv.sums);
    int *cnts = reinterpret_cast<int *>(smem + cv.cnts);
    unsigned char *labels_s = smem + cv.labels;
    unsigned short *queue = reinterpret_cast<unsigned short *>(smem + cv.queue);
    float *mu_s = reinterpret_cast<float *>(smem + cv.misc);              // [32]
    int *shift_s = reinterpret_cast<int *>(smem + cv.misc + 128);         // [32]
    float *cnmax_s = reinterpret_cast<float *>(smem + cv.misc + 256);     // [8]
    int *qcount = reinterpret_cast<int *>(smem + cv.misc + 288);
    int *wide_s = reinterpret_cast<int *>(smem + cv.misc + 576);         // [32] + any at [32]
    double *jpart = reinterpret_cast<double *>(smem + cv.misc + 320);     // [8][4]

    const int tid = threadIdx.x;
    char *wsb = a.ws + (int64_t)b * a.ws_bs;
    const float *Xb = a.X + (int64_t)b * a.x_bs;
    const float *Cb = a.C + (int64_t)b * a.c_bs;

    // group operands and column info into LDS; accumulators to zero
    {
        const float *colmean = reinterpret_cast<const float *>(wsb + a.off_colinfo);
        const int *colshift = reinterpret_cast<const int *>(wsb + a.off_colinfo + 128);
        const int *colwide = reinterpret_cast<const int *>(wsb + a.off_colinfo + 256);
        if (tid < 32) { mu_s[tid] = tid < DP ? colmean[tid] : 0.0f; shift_s[tid] = colshift[tid]; }
        if (tid < 33) wide_s[tid] = colwide[tid];
        const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(wsb + a.off_opA) + (int64_t)g.tile0 * 32 * DP);
        float4 *dst = reinterpret_cast<float4 *>(opA_s);
        for (int e = tid; e < g.n_tiles * 32 * DP / 4; e += kThreads) dst[e] = src[e];
        const float *cnsrc = reinterpret_cast<const float *>(wsb + a.off_cn) + (int64_t)g.tile0 * 32;
        for (int e = tid; e < g.n_tiles * 32; e += kThreads) cn_s[e] = cnsrc[e];
        if (tid < 8) cnmax_s[tid] = tid < g.n_runs ? reinterpret_cast<const float *>(wsb + a.off_cnmax)[g.run0 + tid] : 0.0f;
        if (!FINAL) {
            for (int e = tid; e < real_rows * (DP + 1); e += kThreads) sums[e] = 0ull;
            for (int e = tid; e < real_rows; e += kThreads) cnts[e] = 0;
        }
        if (tid == 0) *qcount = 0;
    }
    __syncthreads();

    const int l = tid % DP, pg = tid / DP;
    const int my_shift = shift_s[l];
    const bool any_wide = wide_s[32] != 0;
    const bool my_wide = wide_s[l] != 0;
    const float eps_a = (float)(DP + 16) * 2.384185791015625e-07f;   // (DP + 16) * 2^-22

    double jloc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) jloc[i] = 0.0;

    const int64_t chunk_begin = (int64_t)chunk * plan.chunk_len;
    const int64_t chunk_end = min(a.N, chunk_begin + plan.chunk_len);

    for (int64_t p0 = chunk_begin; p0 < chunk_end; p0 += TP) {
        const int nvalid = (int)min((int64_t)TP, chunk_end - p0);
        // ---- phase 0: tile load
        long long q[NQ];
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const int p = pg + PPP * i;
            float x = 0.0f;
            if (p < nvalid && l < d) x = Xb[(p0 + p) * a.ldx + l];
            xs[p * XS + l] = x;
            q[i] = to_fixed(x, my_shift);
        }
        __syncthreads();

        // ---- phase A
        switch (g.S) {
        case 1: phase_a<DP, 1>(xs, opA_s, cn_s, mu_s, cnmax_s, labels_s, queue, qcount, g.n_tiles, g.n_runs, nvalid, eps_a); break;
        case 2: phase_a<DP, 2>(xs, opA_s, cn_s, mu_s, cnmax_s, labels_s, queue, qcount, g.n_tiles, g.n_runs, nvalid, eps_a); break;
        case 4: phase_a<DP, 4>(xs, opA_s, cn_s, mu_s, cnmax_s, labels_s, queue, qcount, g.n_tiles, g.n_runs, nvalid, eps_a); break;
        default: phase_a<DP, 8>(xs, opA_s, cn_s, mu_s, cnmax_s, labels_s, queue, qcount, g.n_tiles, g.n_runs, nvalid, eps_a); break;
        }
        __syncthreads();

        // ---- phase B: exact fp64 decision for the queued (point, run) pairs, one pair per wave at a time
        {
            const int nq = *qcount;
            const int lane = tid & 63, wave = tid >> 6;
            for (int e = wave; e < nq; e += kThreads / 64) {
                const int ent = queue[e];
                const int p = ent & 255, rl = ent >> 8;
                const int k = k0 + rl;
                const float *crun = Cb + (int64_t)(rows_before(plan.k_min, g.run0 + rl)) * d;
                double best = INFINITY;
                int arg = 0x7fffffff;
                for (int j = lane; j < k; j += 64) {
                    const double dist = sqdist64(xs + p * XS, crun + (int64_t)j * d, d);
                    if (dist < best) { best = dist; arg = j; }
                }
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    const double ob = __shfl_xor(best, off, 64);
                    const int oa = __shfl_xor(arg, off, 64);
                    if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
                }
                if (lane == 0) labels_s[p * 8 + rl] = (unsigned char)arg;
            }
        }
        __syncthreads();
        if (tid == 0) *qcount = 0;

        // ---- phase C: exact sums (integer adds to the cluster's accumulators)
        if (!FINAL) {
#pragma unroll
            for (int i = 0; i < NQ; ++i) {
                const int p = pg + PPP * i;
                if (p < nvalid && l < d) {
                    const uint2 lab8 = *reinterpret_cast<const uint2 *>(labels_s + p * 8);
                    int rowbase = 0;
                    for (int rl = 0; rl < g.n_runs; ++rl) {
                        const unsigned w = rl < 4 ? lab8.x : lab8.y;
                        const int j = (w >> (8 * (rl & 3))) & 0xff;
                        const int row = rowbase + j;
                        atomicAdd(&sums[row * (DP + 1) + l], (unsigned long long)q[i]);
                        if (l == 0) atomicAdd(&cnts[row], 1);
                        rowbase += k0 + rl;
                    }
                }
            }
            if (any_wide) {
                // rare: values with bits below the column grid add those bits to a global integer accumulator
                long long *losum = reinterpret_cast<long long *>(wsb + a.off_losum);
#pragma unroll 1
                for (int i = 0; i < NQ; ++i) {
                    const int p = pg + PPP * i;
                    if (p < nvalid && l < d && my_wide) {
                        const long long lo = fixed_low(xs[p * XS + l], my_shift);
                        if (lo != 0) {
                            for (int rl = 0; rl < g.n_runs; ++rl) {
                                const int j = labels_s[p * 8 + rl];
                                const int crow = rows_before(plan.k_min, g.run0 + rl) + j;
                                atomicAdd(reinterpret_cast<unsigned long long *>(&losum[(int64_t)crow * d + l]), (unsigned long long)lo);
                            }
                        }
                    }
                }
            }
        }

        // ---- loss of this assignment (fp64, direct form) and label output
        if (LOSS) {
            constexpr int RSTEP = kThreads / TP;      // runs covered per pass: 1 (TP = 256) or 2 (TP = 128)
            const int p = tid % TP;
#pragma unroll
            for (int i = 0; i < 8 / RSTEP; ++i) {
                const int rl = tid / TP + RSTEP * i;
                if (rl < g.n_runs && p < nvalid) {
                    const int j = labels_s[p * 8 + rl];
                    const int crow = rows_before(plan.k_min, g.run0 + rl) + j;
                    jloc[i] = __dadd_rn(jloc[i], sqdist64(xs + p * XS, Cb + (int64_t)crow * d, d));
                    if (FINAL && a.labels)
                        a.labels[(int64_t)b * a.lab_bs + (int64_t)(g.run0 + rl) * a.N + p0 + p] = j;
                }
            }
        }
        __syncthreads();
    }

    if (!FINAL) {
        unsigned long long *psum = reinterpret_cast<unsigned long long *>(wsb + a.off_psum) +
                                   ((int64_t)chunk * plan.total_rows + grow0) * d;
        for (int e = tid; e < real_rows * d; e += kThreads) psum[e] = sums[(e / d) * (DP + 1) + e % d];
        int *pcnt = reinterpret_cast<int *>(wsb + a.off_pcnt) + (int64_t)chunk * plan.total_rows + grow0;
        for (int e = tid; e < real_rows; e += kThreads) pcnt[e] = cnts[e];
    }
    if (LOSS) {
        constexpr int RSTEP = kThreads / TP;
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int i = 0; i < 8 / RSTEP; ++i) {
            double v = jloc[i];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v = __dadd_rn(v, __shfl_xor(v, off, 64));
            if (lane == 0) jpart[i * 4 + wave] = v;
        }
        __syncthreads();
        if (tid < g.n_runs) {
            const int rl = tid;
            double v;
            if (RSTEP == 1) {
                v = __dadd_rn(__dadd_rn(jpart[rl * 4 + 0], jpart[rl * 4 + 1]), __dadd_rn(jpart[rl * 4 + 2], jpart[rl * 4 + 3]));
            } else {
                const int i = rl >> 1, hh = rl & 1;
                v = __dadd_rn(jpart[i * 4 + 2 * hh], jpart[i * 4 + 2 * hh + 1]);
            }
            reinterpret_cast<double *>(wsb + a.off_pj)[(int64_t)chunk * plan.n_runs + g.run0 + rl] = v;
        }
    }
}

// ---- column statistics: mean (for centring), fixed-point shift and range check ----------------
struct ColPart {
    double sum;
    int min_lsb, max_msb, bad, pad;
};

__global__ void __launch_bounds__(kThreads) colstats_kernel(const float *__restrict__ X, int64_t N, int d, int dp, int64_t ldx,
                                                           int64_t x_bs, char *ws, int64_t ws_bs, int64_t off_part)
{
    __shared__ ColPart sh[kThreads];
    const int b = blockIdx.y;
    const float *Xb = X + (int64_t)b * x_bs;
    const int tid = threadIdx.x;
    const int l = tid % dp, pg = tid / dp, ppp = kThreads / dp;
    const int64_t per = (N + gridDim.x - 1) / gridDim.x;
    const int64_t r0 = (int64_t)blockIdx.x * per, r1 = min(N, r0 + per);
    ColPart c = {0.0, 1 << 20, -(1 << 20), 0, 0};
    if (l < d) {
        for (int64_t r = r0 + pg; r < r1; r += ppp) {
            const float x = Xb[r * ldx + l];
            const unsigned u = __float_as_uint(x);
            int e = (int)((u >> 23) & 0xffu);
            unsigned m = u & 0x7fffffu;
            if (e == 255) { c.bad = 1; continue; }
            c.sum = __dadd_rn(c.sum, (double)x);
            if (e == 0) { if (m == 0) continue; e = 1; } else m |= 0x800000u;
            const int lsb = e - 150 + (__ffs((int)m) - 1);
            const int msb = e - 150 + (31 - __clz((int)m));
            c.min_lsb = min(c.min_lsb, lsb);
            c.max_msb = max(c.max_msb, msb);
        }
    }
    sh[tid] = c;
    __syncthreads();
    if (tid < dp) {
        ColPart t = sh[tid];
        for (int g = 1; g < ppp; ++g) {
            const ColPart o = sh[g * dp + tid];
            t.sum = __dadd_rn(t.sum, o.sum);
            t.min_lsb = min(t.min_lsb, o.min_lsb);
            t.max_msb = max(t.max_msb, o.max_msb);
            t.bad |= o.bad;
        }
        reinterpret_cast<ColPart *>(ws + (int64_t)b * ws_bs + off_part)[blockIdx.x * 32 + tid] = t;
    }
}

__global__ void colstats_final_kernel(int64_t N, int d, int n_blocks, char *ws, int64_t ws_bs, int64_t off_part,
                                      int64_t off_colinfo, int32_t *status)
{
    __shared__ int flags;
    const int b = blockIdx.x, l = threadIdx.x;   // 32 threads
    if (l == 0) flags = 0;
    __syncthreads();
    const ColPart *part = reinterpret_cast<const ColPart *>(ws + (int64_t)b * ws_bs + off_part);
    float mean = 0.0f;
    int shift = 0, wide = 0;
    if (l < d) {
        ColPart t = part[l];
        for (int g = 1; g < n_blocks; ++g) {
            const ColPart o = part[g * 32 + l];
            t.sum = __dadd_rn(t.sum, o.sum);
            t.min_lsb = min(t.min_lsb, o.min_lsb);
            t.max_msb = max(t.max_msb, o.max_msb);
            t.bad |= o.bad;
        }
        if (t.bad) atomicOr(&flags, RLS_STATUS_NONFINITE);
        else {
            mean = (float)(t.sum / (double)N);
            if (t.max_msb >= t.min_lsb) {
                // grid: the finest bit kept by the main accumulator. |x * 2^shift| < 2^kGridBits, and a chunk adds
                // at most 2^17 of them into 63 bits. Bits below the grid (wide columns) go to the low accumulator,
                // which keeps kLowBits more; anything finer cannot be summed exactly.
                int grid = t.max_msb - (kGridBits - 1);
                if (grid < t.min_lsb) grid = t.min_lsb;
                shift = -grid;
                if (t.min_lsb < grid) wide = 1;
                if (t.min_lsb < grid - kLowBits) atomicOr(&flags, RLS_STATUS_RANGE);
            }
        }
    }
    float *colmean = reinterpret_cast<float *>(ws + (int64_t)b * ws_bs + off_colinfo);
    int *colshift = reinterpret_cast<int *>(ws + (int64_t)b * ws_bs + off_colinfo + 128);
    int *colwide = reinterpret_cast<int *>(ws + (int64_t)b * ws_bs + off_colinfo + 256);
    colmean[l] = mean;
    colshift[l] = shift;
    colwide[l] = wide;
    if (wide) atomicOr(&flags, 1 << 16);
    __syncthreads();
    if (l == 0) { colwide[32] = (flags >> 16) & 1; status[b] = flags & 0xffff; }
}

// ---- operand fill: padding rows are zero vectors with a huge norm ----------------------------
__global__ void fill_operands_kernel(char *ws, int64_t ws_bs, int64_t off_opA, int64_t off_cn, int64_t n_opA, int64_t n_cn,
                                     int64_t off_losum, int64_t n_losum)
{
    long long *losum = reinterpret_cast<long long *>(ws + (int64_t)blockIdx.y * ws_bs + off_losum);
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_losum; e += (int64_t)gridDim.x * blockDim.x) losum[e] = 0;
    float *opA = reinterpret_cast<float *>(ws + (int64_t)blockIdx.y * ws_bs + off_opA);
    float *cn = reinterpret_cast<float *>(ws + (int64_t)blockIdx.y * ws_bs + off_cn);
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_opA; e += (int64_t)gridDim.x * blockDim.x) opA[e] = 0.0f;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_cn; e += (int64_t)gridDim.x * blockDim.x) cn[e] = kPadNorm;
}

// 128-bit two's complement sum (hi, lo) -> fp64 with one round-to-nearest-even, scaled by 2^-shift
__device__ inline double fixed128_to_double(long long hi, unsigned long long lo, int shift)
{
    const bool neg = hi < 0;
    unsigned long long mh = (unsigned long long)hi, ml = lo;
    if (neg) {
        ml = ~ml + 1ull;
        mh = ~mh + (ml == 0ull ? 1ull : 0ull);
    }
    double mag;
    if (mh == 0ull && (ml >> 53) == 0ull) {
        mag = (double)ml;                       // exact
        mag = ldexp(mag, -shift);
    } else {
        const int nbits = mh ? 128 - __clzll((long long)mh) : 64 - __clzll((long long)ml);
        const int sh = nbits - 53;              // >= 1
        // top = mag >> sh (53 bits), rem = mag & (2^sh - 1)
        unsigned long long top, rem_hi, rem_lo;
        if (sh >= 64) {
            top = mh >> (sh - 64);
            rem_hi = sh == 64 ? 0ull : (mh & ((1ull << (sh - 64)) - 1ull));
            rem_lo = ml;
        } else {
            top = (ml >> sh) | (mh ? (mh << (64 - sh)) : 0ull);
            rem_hi = 0ull;
            rem_lo = ml & ((1ull << sh) - 1ull);
        }
        // compare remainder with half = 2^(sh-1)
        int cmp;   // -1 below half, 0 equal, 1 above
        if (sh > 64) {
            const unsigned long long half_hi = 1ull << (sh - 65);
            cmp = rem_hi > half_hi ? 1 : (rem_hi < half_hi ? -1 : (rem_lo ? 1 : 0));
        } else if (sh == 64) {
            const unsigned long long half_lo = 1ull << 63;
            cmp = rem_lo > half_lo ? 1 : (rem_lo < half_lo ? -1 : 0);
        } else {
            const unsigned long long half_lo = 1ull << (sh - 1);
            cmp = rem_lo > half_lo ? 1 : (rem_lo < half_lo ? -1 : 0);
        }
        if (cmp > 0 || (cmp == 0 && (top & 1ull))) top += 1ull;
        mag = ldexp((double)top, sh - shift);   // top <= 2^53: exact
    }
    return neg ? -mag : mag;
}

struct CentroidArgs {
    const float *X;
    int64_t N;
    int32_t d;
    int64_t ldx, x_bs;
    const int64_t *init_idx;     // [batch][init_bs] (INIT only)
    int64_t init_bs;
    float *C;
    int64_t c_bs;
    const int32_t *status;
    char *ws;
    int64_t ws_bs;
    int64_t off_colinfo, off_opA, off_cn, off_cnmax, off_psum, off_pcnt, off_losum;
};

// One workgroup per run: new centroids (from the seeding rows, or from the per-chunk partial sums),
// then the centred, -2-scaled MFMA operand rows and their squared norms.
template <int DP, bool INIT>
__global__ void __launch_bounds__(kThreads) lloyd_centroids_kernel(SweepPlan plan, CentroidArgs a)
{
    __shared__ float cs[RLS_MAX_K * DP];     // centred centroids of this run
    __shared__ float wmax[kThreads / 64];
    const int b = blockIdx.y, run = blockIdx.x, tid = threadIdx.x;
    if (a.status[b] != 0) return;
    const int d = a.d, k = plan.k_min + run;
    const int row0 = rows_before(plan.k_min, run);
    int gi = 0;
    while (gi + 1 < plan.n_groups && plan.g[gi + 1].run0 <= run) ++gi;
    const GroupDesc g = plan.g[gi];
    const int rl = run - g.run0;
    char *wsb = a.ws + (int64_t)b * a.ws_bs;
    const float *colmean = reinterpret_cast<const float *>(wsb + a.off_colinfo);
    const int *colshift = reinterpret_cast<const int *>(wsb + a.off_colinfo + 128);
    const int *colwide = reinterpret_cast<const int *>(wsb + a.off_colinfo + 256);
    float *Cb = a.C + (int64_t)b * a.c_bs;
    float *opA = reinterpret_cast<float *>(wsb + a.off_opA) + (int64_t)g.tile0 * 32 * DP;
    float *cn = reinterpret_cast<float *>(wsb + a.off_cn) + (int64_t)g.tile0 * 32;

    for (int e = tid; e < k * DP; e += kThreads) {
        const int j = e / DP, l = e % DP;
        float cp = 0.0f;
        if (l < d) {
            float c;
            if (INIT) {
                const int64_t src = a.init_idx[(int64_t)b * a.init_bs + j];
                c = a.X[(int64_t)b * a.x_bs + src * a.ldx + l];
                Cb[(int64_t)(row0 + j) * d + l] = c;
            } else {
                const long long *psum = reinterpret_cast<const long long *>(wsb + a.off_psum);
                const int *pcnt = reinterpret_cast<const int *>(wsb + a.off_pcnt);
                long long hi = 0;
                unsigned long long lo = 0;
                long long cnt = 0;
                for (int c0 = 0; c0 < plan.n_chunks; ++c0) {
                    const long long v = psum[((int64_t)c0 * plan.total_rows + row0 + j) * d + l];
                    const unsigned long long nlo = lo + (unsigned long long)v;
                    hi += (v >> 63) + (nlo < lo ? 1 : 0);
                    lo = nlo;
                    cnt += pcnt[(int64_t)c0 * plan.total_rows + row0 + j];
                }
                int shift = colshift[l];
                if (colwide[l]) {
                    // total = main * 2^kLowBits + low, on the scale 2^-(shift + kLowBits)
                    long long *losum = reinterpret_cast<long long *>(wsb + a.off_losum) + (int64_t)(row0 + j) * d + l;
                    const long long low = *losum;
                    *losum = 0;
                    hi = (long long)(((unsigned long long)hi << kLowBits) | (lo >> (64 - kLowBits)));
                    lo = lo << kLowBits;
                    const unsigned long long nlo = lo + (unsigned long long)low;
                    hi += (low >> 63) + (nlo < lo ? 1 : 0);
                    lo = nlo;
                    shift += kLowBits;
                }
                if (cnt > 0) {
                    c = (float)(fixed128_to_double(hi, lo, shift) / (double)cnt);
                    Cb[(int64_t)(row0 + j) * d + l] = c;
                } else {
                    c = Cb[(int64_t)(row0 + j) * d + l];     // a cluster without members keeps its centroid
                }
            }
            cp = c - colmean[l];
        }
        cs[j * DP + l] = cp;
        // operand position of (centroid j, feature l)
        const int qd = j >> 2, i = j & 3;
        const int t = qd / g.S, slot = rl * g.S + qd % g.S;
        const int m = 8 * (slot & 3) + 4 * (slot >> 2) + i;
        const int h = l / (DP / 2), s = l % (DP / 2);
        opA[((((t * 2 + h) * (DP / 8) + (s >> 2)) * 32 + m) << 2) + (s & 3)] = -2.0f * cp;
    }
    __syncthreads();
    float mx = 0.0f;
    for (int j = tid; j < k; j += kThreads) {
        float nrm = 0.0f;
        for (int l = 0; l < DP; ++l) nrm = fmaf(cs[j * DP + l], cs[j * DP + l], nrm);
        const int qd = j >> 2, i = j & 3;
        const int t = qd / g.S, slot = rl * g.S + qd % g.S;
        cn[t * 32 + 8 * (slot & 3) + 4 * (slot >> 2) + i] = nrm;
        mx = fmaxf(mx, nrm);
    }
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if ((tid & 63) == 0) wmax[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) {
        float m = wmax[0];
        for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, wmax[w]);
        reinterpret_cast<float *>(wsb + a.off_cnmax)[run] = m;
    }
}

// sum of the per-chunk partial losses of every run, in chunk order
__global__ void lloyd_loss_kernel(int n_runs, int n_chunks, const int32_t *status, const char *ws, int64_t ws_bs,
                                  int64_t off_pj, double *out, int64_t out_bs, int64_t out_stride, int64_t out_off)
{
    const int b = blockIdx.x, r = threadIdx.x;
    if (r >= n_runs || status[b] != 0) return;
    const double *pj = reinterpret_cast<const double *>(ws + (int64_t)b * ws_bs + off_pj);
    double v = 0.0;
    for (int c = 0; c < n_chunks; ++c) v = __dadd_rn(v, pj[(int64_t)c * n_runs + r]);
    out[(int64_t)b * out_bs + (int64_t)r * out_stride + out_off] = v;
}

template <int DP>
hipError_t launch_sweep_dp(const SweepPlan &plan, const SweepLayout &L, const SweepArgs &a, hipStream_t s)
{
    static bool attr_set = false;
    if (!attr_set) {
        const void *fns[] = {
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, false, false>),
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, false, true>),
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, true, false>),
        };
        for (const void *fn : fns) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const int batch = a.batch;
    // column statistics
    hipLaunchKernelGGL(colstats_kernel, dim3(L.stat_blocks, batch), dim3(kThreads), 0, s, a.X, a.N, (int)a.d, DP, a.ldx,
                       a.x_batch_stride, a.ws, L.per_batch, L.colstat_part);
    hipLaunchKernelGGL(colstats_final_kernel, dim3(batch), dim3(32), 0, s, a.N, (int)a.d, (int)L.stat_blocks, a.ws,
                       L.per_batch, L.colstat_part, L.colinfo, a.status);
    hipLaunchKernelGGL(fill_operands_kernel, dim3(64, batch), dim3(256), 0, s, a.ws, L.per_batch, L.opA, L.cn,
                       (int64_t)plan.total_tiles * 32 * DP, (int64_t)plan.total_tiles * 32, L.losum,
                       (int64_t)plan.total_rows * a.d);

    CentroidArgs ca;
    ca.X = a.X; ca.N = a.N; ca.d = a.d; ca.ldx = a.ldx; ca.x_bs = a.x_batch_stride;
    ca.init_idx = a.init_idx; ca.init_bs = a.init_batch_stride;
    ca.C = a.centroids; ca.c_bs = (int64_t)plan.total_rows * a.d;
    ca.status = a.status; ca.ws = a.ws; ca.ws_bs = L.per_batch;
    ca.off_colinfo = L.colinfo; ca.off_opA = L.opA; ca.off_cn = L.cn; ca.off_cnmax = L.cnmax;
    ca.off_psum = L.psum; ca.off_pcnt = L.pcnt; ca.off_losum = L.losum;
    hipLaunchKernelGGL((lloyd_centroids_kernel<DP, true>), dim3(plan.n_runs, batch), dim3(kThreads), 0, s, plan, ca);

    StepArgs sa;
    sa.X = a.X; sa.N = a.N; sa.d = a.d; sa.ldx = a.ldx; sa.x_bs = a.x_batch_stride;
    sa.C = a.centroids; sa.c_bs = ca.c_bs;
    sa.labels = a.labels; sa.lab_bs = (int64_t)plan.n_runs * a.N;
    sa.status = a.status; sa.ws = a.ws; sa.ws_bs = L.per_batch;
    sa.off_colinfo = L.colinfo; sa.off_opA = L.opA; sa.off_cn = L.cn; sa.off_cnmax = L.cnmax;
    sa.off_psum = L.psum; sa.off_pcnt = L.pcnt; sa.off_pj = L.pj; sa.off_losum = L.losum;

    size_t lds = 0;
    for (int gi = 0; gi < plan.n_groups; ++gi) {
        const GroupDesc &g = plan.g[gi];
        const int rr = rows_before(plan.k_min, g.run0 + g.n_runs) - rows_before(plan.k_min, g.run0);
        const size_t need = (size_t)carve_lds(DP, g.n_tiles, rr).total;
        if (need > lds) lds = need;
    }
    const dim3 grid(plan.n_groups * plan.n_chunks, batch);
    const bool trace = a.trace != nullptr;
    for (int t = 0; t < a.iters; ++t) {
        if (trace) {
            hipLaunchKernelGGL((lloyd_step_kernel<DP, false, true>), grid, dim3(kThreads), lds, s, plan, sa);
            hipLaunchKernelGGL(lloyd_loss_kernel, dim3(batch), dim3(128), 0, s, plan.n_runs, plan.n_chunks, a.status, a.ws,
                               L.per_batch, L.pj, a.trace, (int64_t)plan.n_runs * (a.iters + 1), (int64_t)(a.iters + 1), (int64_t)t);
        } else {
            hipLaunchKernelGGL((lloyd_step_kernel<DP, false, false>), grid, dim3(kThreads), lds, s, plan, sa);
        }
        hipLaunchKernelGGL((lloyd_centroids_kernel<DP, false>), dim3(plan.n_runs, batch), dim3(kThreads), 0, s, plan, ca);
    }
    hipLaunchKernelGGL((lloyd_step_kernel<DP, true, false>), grid, dim3(kThreads), lds, s, plan, sa);
    hipLaunchKernelGGL(lloyd_loss_kernel, dim3(batch), dim3(128), 0, s, plan.n_runs, plan.n_chunks, a.status, a.ws, L.per_batch,
                       L.pj, a.inertia, (int64_t)plan.n_runs, (int64_t)1, (int64_t)0);
    if (trace)
        hipLaunchKernelGGL(lloyd_loss_kernel, dim3(batch), dim3(128), 0, s, plan.n_runs, plan.n_chunks, a.status, a.ws,
                           L.per_batch, L.pj, a.trace, (int64_t)plan.n_runs * (a.iters + 1), (int64_t)(a.iters + 1),
                           (int64_t)a.iters);
    return hipGetLastError();
}

}  // namespace

int padded_d(int d) { return d <= 8 ? 8 : (d <= 16 ? 16 : 32); }

LloydGeometry lloyd_geometry(int dp)
{
    LloydGeometry g;
    g.threads = kThreads;
    g.tile_points = tile_points_of(dp);
    g.lds_budget = 80 * 1024;
    return g;
}

int64_t lloyd_group_lds_bytes(int dp, int tile_points, int n_tiles, int real_rows)
{
    (void)tile_points;
    return carve_lds(dp, n_tiles, real_rows).total;
}

int32_t make_sweep_plan(int64_t N, int32_t d, int32_t k_min, int32_t k_max, SweepPlan *plan)
{
    const int dp = padded_d(d);
    const LloydGeometry geo = lloyd_geometry(dp);
    plan->n_runs = k_max - k_min + 1;
    plan->k_min = k_min;
    plan->dp = dp;
    plan->n_groups = 0;
    int tiles = 0;
    int run = 0;
    while (run < plan->n_runs) {
        bool placed = false;
        for (int R = 8; R >= 1 && !placed; R >>= 1) {
            const int S = 8 / R;
            const int nr = plan->n_runs - run < R ? plan->n_runs - run : R;
            const int kmax_g = k_min + run + nr - 1;
            const int quads = (kmax_g + 3) / 4;
            const int n_tiles = (quads + S - 1) / S;
            const int real_rows = rows_before(k_min, run + nr) - rows_before(k_min, run);
            if (n_tiles > 32) continue;
            if (lloyd_group_lds_bytes(dp, geo.tile_points, n_tiles, real_rows) > geo.lds_budget) continue;
            if (plan->n_groups >= kMaxGroups) return RLS_ERR_INVALID_ARG;
            GroupDesc &g = plan->g[plan->n_groups++];
            g.run0 = (int16_t)run; g.n_runs = (int16_t)nr; g.S = (int16_t)S; g.n_tiles = (int16_t)n_tiles; g.tile0 = tiles;
            tiles += n_tiles;
            run += nr;
            placed = true;
        }
        if (!placed) return RLS_ERR_INVALID_ARG;
    }
    plan->total_tiles = tiles;
    plan->total_rows = rows_before(k_min, plan->n_runs);
    // chunks: enough workgroups to fill the chip several times over; a chunk never exceeds 2^17 points
    const int tp = geo.tile_points;
    const int64_t tiles_total = (N + tp - 1) / tp;
    int64_t want = (4096 + plan->n_groups - 1) / plan->n_groups;
    if (want > tiles_total) want = tiles_total;
    if (want < 1) want = 1;
    int64_t chunk_len = ((tiles_total + want - 1) / want) * tp;
    const int64_t cap = (int64_t)1 << 17;
    if (chunk_len > cap) chunk_len = cap / tp * tp;
    plan->chunk_len = (int32_t)chunk_len;
    plan->n_chunks = (int32_t)((N + chunk_len - 1) / chunk_len);
    return RLS_OK;
}

void sweep_layout(const SweepPlan &plan, int64_t N, int32_t d, int32_t k_max, int32_t batch, SweepLayout *L)
{
    int64_t off = 0;
    auto take = [&](int64_t bytes) { const int64_t o = off; off += align_up(bytes, 256); return o; };
    L->stat_blocks = (int32_t)(N < 65536 ? (N + 255) / 256 : kStatBlocks);
    if (L->stat_blocks > kStatBlocks) L->stat_blocks = kStatBlocks;
    if (L->stat_blocks < 1) L->stat_blocks = 1;
    L->seed_blocks = (int32_t)((N + kSeedBlock - 1) / kSeedBlock);
    L->colstat_part = take((int64_t)kStatBlocks * 32 * sizeof(ColPart));
    L->colinfo = take(512);
    L->chain = take((int64_t)k_max * 8);
    L->mind = take(N * 8);
    L->bsum = take((int64_t)L->seed_blocks * 8);
    L->opA = take((int64_t)plan.total_tiles * 32 * plan.dp * 4);
    L->cn = take((int64_t)plan.total_tiles * 32 * 4);
    L->cnmax = take((int64_t)plan.n_runs * 4);
    L->psum = take((int64_t)plan.n_chunks * plan.total_rows * d * 8);
    L->pcnt = take((int64_t)plan.n_chunks * plan.total_rows * 4);
    L->pj = take((int64_t)plan.n_chunks * plan.n_runs * 8);
    L->losum = take((int64_t)plan.total_rows * d * 8);
    L->per_batch = off;
    L->total = off * batch;
}

hipError_t launch_sweep(const SweepPlan &plan, const SweepLayout &L, const SweepArgs &a, hipStream_t s)
{
    switch (plan.dp) {
    case 8: return launch_sweep_dp<8>(plan, L, a, s);
    case 16: return launch_sweep_dp<16>(plan, L, a, s);
    default: return launch_sweep_dp<32>(plan, L, a, s);
    }
}

}  // namespace rls
