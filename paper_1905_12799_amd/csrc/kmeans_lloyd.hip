// Lloyd's k-means for every k of a range at once: the "k-means(s_Theta, k)" call inside the loop of
// Algorithm 1 (Sec. 4.2 of the paper), all k side by side, iterations in lock step.
//
// Per iteration one launch of lloyd_step_kernel covers every (group of runs, chunk of points).  A workgroup
// stages its group's operand rows, a copy of its centroids and integer accumulators in LDS once; then each of
// its waves (twelve up to d_pad = 16, eight at 32) works through its own points without any barrier:
//   load     each lane loads its half of the features of its points straight into registers, one step ahead; from
//            the second round on the lanes load the matrix operands themselves, which lloyd_prepare_kernel derives
//            once per sweep from the rows (centred, scaled, split into fp16 pieces, squared norm), and a raw row
//            is read again only for a point that needs it: a close call or a changed label
//   assign   distances in the expansion |c'|^2 + |x'|^2 - 2 x'.c' on data centred by the column means and scaled
//            by one power of two into fp16 range, on the 16-bit matrix pipeline: every fp32 operand is split
//            into two fp16 pieces (22 significant bits) and the three leading cross products are accumulated
//            in fp32 (fp32-class accuracy; the 16-bit pipeline runs beside the vector ALU, the fp32 one does
//            not); per point and run the two smallest packed (value, index) keys are kept.  When they are
//            closer than the error bound of these distances the pair is decided again with the direct
//            form sum_l (x_l - c_l)^2 - the arithmetic that defines the assignment - by a scan of the whole
//            run: in fp32 first, whose relative error bound leaves a single candidate almost always, then in
//            fp64 among several; labels never depend on the rounding of the matrix-pipeline distances
//   update   exact centroid sums, kept as running totals: only points whose label differs from the one
//            of the previous round (kept as one byte per point and run, the runs of a group side by side, so
//            that a lane compares all its runs in one instruction) move their fixed-point row from the old cluster's int64 accumulators
//            to the new one's (integer LDS atomics; integer adds commute and cancel exactly, so the totals
//            equal a fresh sum in any order); per-chunk deltas go to global memory and lloyd_centroids_kernel
//            adds them to the 128-bit totals, rounds once to fp64, divides by the count and rounds to fp32
// The final pass replaces the update by the fp64 loss of every point and the label output.
#include <mutex>
#include <type_traits>

#include "rls_internal.h"

namespace rls {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int kThreads = 512;                // workgroup of the helper kernels (the step kernel: step_threads_of)
constexpr int kPartRows = 8;                 // centroids of a run that one workgroup of the centroid kernel renews
constexpr int kMaxParts = RLS_MAX_K / kPartRows;
// parts of the runs k' = 1 .. k together: the sum of ceil(k' / kPartRows)
__host__ __device__ inline int parts_upto(int k)
{
    const int q = k / kPartRows;
    return kPartRows * q * (q + 1) / 2 + (k - kPartRows * q) * (q + 1);
}
constexpr float kPadNorm = 1.0e30f;           // squared norm given to padding rows: never the minimum
constexpr int kBigKey = 0x7f000000;           // larger than any key of a finite distance below 1.7e38
constexpr int kGridBits = 44;                 // bits of |x * 2^shift| kept by the main accumulator
constexpr int kLowBits = 36;                  // further bits kept by the low accumulator (wide columns)
// The centred data is scaled by a power of two so that |x'| < 2^13 and |2 c'| < 2^14 sit well inside fp16; an fp16
// piece below 2^-14 (subnormal) may be lost, which costs a distance at most 0.078 d + S 2^-24 in scaled units (see eps_a)
constexpr int kScaledMsb = 14;
constexpr float kTolFloor = 8.0f;             // twice that loss at d = 32, in scaled squared units
constexpr int kColScaleOff = 400;             // byte offset of the scale factor in the column info block

__host__ __device__ constexpr int tile_points_of(int dp) { return dp == 32 ? 256 : 512; }
// 32-point blocks a wave takes per slab.  Up to d_pad = 16: one, which keeps a wave under 168 registers so that three
// waves fit a SIMD (measured: 6% shorter launches than two waves with two blocks each).  At d_pad = 32 three waves do
// not fit; there a wave takes two blocks, except with eight runs side by side, where the best keys of 4 runs x 2 blocks
// would not fit the registers next to the operands.
__host__ __device__ constexpr int slab_blocks_of(int dp, int s) { return dp <= 16 ? 1 : (s < 2 ? 1 : 2); }
// threads of a step workgroup: up to d_pad = 16 one block per slab leaves room for three waves per SIMD
__host__ __device__ constexpr int step_threads_of(int dp) { return dp <= 16 ? 768 : 512; }
// MFMA operands: a lane holds 8 fp16 values of its half of the features per K-step (v_mfma_f32_32x32x16_f16);
// a 32-row tile stores, per K-step, the two pieces (high, low) of -2c', and then one bias slot (bf16).
__host__ __device__ constexpr int ksteps_of(int dp) { return dp == 32 ? 2 : 1; }
__host__ __device__ constexpr int tile_slots_of(int dp) { return 2 * ksteps_of(dp) + 1; }          // 16-byte slots per lane
__host__ __device__ constexpr int tile_bytes_of(int dp) { return tile_slots_of(dp) * 64 * 16; }    // per 32-row tile

// Prepared copy of the points (written once per sweep by lloyd_prepare_kernel): per block of 32 points the B operands
// of the distance tiles in the lane order of the step kernel - 2 * ksteps slots (high pieces, then low pieces, per
// K-step) of 64 lanes x 16 bytes - followed by 32 entries of 8 bytes with the point's squared norm as the three bf16
// pieces the bias slot wants (their sum, which is the norm cut off below 2^-24 of itself, serves the error bound).
__host__ __device__ constexpr int prep_slots_of(int dp) { return 2 * ksteps_of(dp); }
__host__ __device__ constexpr int prep_block_u4_of(int dp) { return prep_slots_of(dp) * 64 + 16; }   // 16-byte units per block
// Moved pairs of the rounds that run on the prepared copy: every wave keeps a ring of records in global memory
// (point within the chunk, accumulator row of the new label | row of the old label) and works it off 64 records at a time.
constexpr int kLogCap = 512;                  // records per wave (a slab adds at most 4 x 64; 63 may be left over)

// ---- LDS carve of lloyd_step_kernel (bytes), shared by the planner and the kernel ------------
struct Carve {
    int opA, cs, sums, cnts, misc, total;
};
__host__ __device__ inline Carve carve_lds(int dp, int d, int n_tiles, int real_rows, int copies)
{
    Carve c;
    int off = 0;
    c.opA = off;     off += n_tiles * tile_bytes_of(dp);       // MFMA operand rows of the group (fp16 pieces + bias slot)
    c.cs = off;      off += real_rows * (dp + 4) * 4;                   // centroids as given, rows of dp + 4 floats, zero-padded
    // accumulators: `copies` of them side by side (a lane adds to copy lane % copies, which spreads the lanes that
    // hit one cluster of a run with few clusters over several addresses; the copies are summed at the end)
    c.sums = off;    off += copies * real_rows * (dp + 1) * 8;          // fixed-point sum deltas
    c.cnts = off;    off += (copies * real_rows * 4 + 15) / 16 * 16;    // member count deltas
    c.misc = off;    off += 2048;
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
    int64_t off_colinfo, off_opA, off_cnmax, off_psum, off_pcnt, off_pj, off_losum, off_prev, off_xp, off_log;
    int32_t first_round;     // 1: no point has a label yet (every pair enters a cluster, nothing leaves one)
    int32_t batch;           // spaces swept by the launch
};

// x * 2^shift truncated toward zero, |x * 2^shift| < 2^kGridBits; exact whenever x is a multiple of 2^-shift.
// The scaling is exact in fp64; adding 2^52 + 2^51 leaves the integer in the low bits of the significand.
__device__ inline long long to_fixed(float x, int shift)
{
    const double t = trunc(ldexp((double)x, shift));
    return __double_as_longlong(__dadd_rn(t, 6755399441055744.0)) - 0x4338000000000000ll;
}

// The accumulators hold "biased" fixed-point rows: the bit pattern of the double 2^52 + 2^51 + x * 2^shift, which is
// kFixBias plus the two's complement integer x * 2^shift.  A row that enters a cluster adds its patterns, a row that
// leaves subtracts them, so an accumulator is off by kFixBias times the net number of rows - the member count delta,
// which is tracked anyway - and the bias is taken out once per chunk.  For a column whose values are all multiples of
// 2^-shift the product is an exact integer and one fused multiply-add (by the power of two 2^shift, whose high word
// comes from LDS) yields the pattern: two vector instructions per feature.
constexpr unsigned long long kFixBias = 0x4338000000000000ull;
__device__ inline unsigned long long fixed_biased(float x, int pow2_hi)
{
    return (unsigned long long)__double_as_longlong(fma((double)x, __hiloint2double(pow2_hi, 0), 6755399441055744.0));
}

// The part of x below the column grid 2^-shift, scaled by 2^(shift + kLowBits): the bits that to_fixed drops.
// Non-zero only in columns whose values span more than kGridBits binary digits.
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

// value of the lane 32 places away (the other half-wave), by a register swap: no trip through LDS
__device__ inline int xchg32(int v)
{
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ inline unsigned xchg32(unsigned v) { return (unsigned)xchg32((int)v); }
__device__ inline float xchg32(float v) { return __int_as_float(xchg32(__float_as_int(v))); }

// Minimum over the wave, in every lane, without a trip through LDS: lane exchanges inside rows of 16 by DPP (swap
// neighbours, swap pairs, mirror halves of 8, mirror the row: after each step twice as many lanes agree), then
// between rows with the two row-swap instructions.
template <int CTRL>
__device__ inline int dpp_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }   // every lane has a source
template <int CTRL>
__device__ inline double dpp_move(double v)
{
    return __hiloint2double(dpp_move<CTRL>(__double2hiint(v)), dpp_move<CTRL>(__double2loint(v)));
}
constexpr int kDppSwap1 = 0xB1, kDppSwap2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;
__device__ inline double wave_min_f64(double v)
{
    v = fmin(v, dpp_move<kDppSwap1>(v));
    v = fmin(v, dpp_move<kDppSwap2>(v));
    v = fmin(v, dpp_move<kDppHalfMirror>(v));
    v = fmin(v, dpp_move<kDppMirror>(v));
    {
        const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        v = fmin(__hiloint2double((int)rh[0], (int)rl[0]), __hiloint2double((int)rh[1], (int)rl[1]));   // own row, other row
    }
    {
        const unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
        const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        v = fmin(__hiloint2double((int)rh[0], (int)rl[0]), __hiloint2double((int)rh[1], (int)rl[1]));
    }
    return v;
}
__device__ inline int wave_min_i32(int v)
{
    v = min(v, dpp_move<kDppSwap1>(v));
    v = min(v, dpp_move<kDppSwap2>(v));
    v = min(v, dpp_move<kDppHalfMirror>(v));
    v = min(v, dpp_move<kDppMirror>(v));
    {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        v = min((int)r[0], (int)r[1]);
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        v = min((int)r[0], (int)r[1]);
    }
    return v;
}

__device__ inline float wave_min_f32(float v)
{
    v = fminf(v, __int_as_float(dpp_move<kDppSwap1>(__float_as_int(v))));
    v = fminf(v, __int_as_float(dpp_move<kDppSwap2>(__float_as_int(v))));
    v = fminf(v, __int_as_float(dpp_move<kDppHalfMirror>(__float_as_int(v))));
    v = fminf(v, __int_as_float(dpp_move<kDppMirror>(__float_as_int(v))));
    {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = fminf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}

// The assignment as it is defined, by one whole wave: fp64 direct-form distances sum_l (x_l - c_l)^2, features in
// rising order, of one point to the k centroids of a run (one or two per lane), then the lexicographic minimum of
// (distance, index) over the wave.  Every lane returns the winner.  The point arrives as wave-uniform values (read
// out of the registers of the two lanes that hold its halves); the centroid rows come from the LDS copy, which is
// zero beyond the last feature, as is the register copy of the point: padded terms add +0.
//
// Almost every call is settled by a first stage in fp32: the same direct form (difference, square, sum; all terms
// are non-negative, so nothing cancels) is within (DP + 2) 2^-24 of the real-number distance, relatively, and the
// fp64 form within (DP + 2) 2^-53.  A centroid whose fp32 distance exceeds the smallest one by more than 8 (DP + 2)
// 2^-24 of it (more than twice the two errors and the rounding of the threshold itself) cannot have the smallest
// fp64 distance; when a single centroid is left it is the winner.  Several left (true ties, duplicated centroids),
// or a smallest distance so small or large that fp32 may have lost it (below 1e-30, infinite): fp64 over the whole run.
template <int DP>
__device__ inline int exact_argmin_wave(const float (&x)[DP], const float *crun, int cstride, int k)
{
    const int lane = threadIdx.x & 63;
    {
        float d32[2] = {INFINITY, INFINITY};        // this lane's centroids: lane and lane + 64 (k <= 128)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = lane + 64 * u;
            if (u == 1 && k <= 64) break;           // wave-uniform
            const float *crow = crun + min(j, k - 1) * cstride;
            float acc = 0.0f;
#pragma unroll
            for (int l = 0; l < DP; l += 4) {
                const float4 cv = *reinterpret_cast<const float4 *>(crow + l);
                float diff = x[l] - cv.x;
                acc = fmaf(diff, diff, acc);
                diff = x[l + 1] - cv.y;
                acc = fmaf(diff, diff, acc);
                diff = x[l + 2] - cv.z;
                acc = fmaf(diff, diff, acc);
                diff = x[l + 3] - cv.w;
                acc = fmaf(diff, diff, acc);
            }
            if (j < k) d32[u] = acc;
        }
        const float wmin = wave_min_f32(fminf(d32[0], d32[1]));
        const float thr = fmaf(wmin, (float)(8 * (DP + 2)) * 5.9604644775390625e-08f, wmin);
        const unsigned long long c0 = __ballot(d32[0] <= thr), c1 = __ballot(d32[1] <= thr);
        if (__popcll(c0) + __popcll(c1) == 1 && wmin >= 1.0e-30f && wmin < INFINITY)
            return c0 ? __ffsll((long long)c0) - 1 : 63 + __ffsll((long long)c1);
    }
    double best = INFINITY;
    int arg = 0x7fffffff;
    for (int j = lane; j < k; j += 64) {
        const float *crow = crun + j * cstride;
        double dist = 0.0;
#pragma unroll
        for (int l = 0; l < DP; l += 4) {
            const float4 cv = *reinterpret_cast<const float4 *>(crow + l);
            double diff = __dsub_rn((double)x[l], (double)cv.x);
            dist = __dadd_rn(dist, __dmul_rn(diff, diff));
            diff = __dsub_rn((double)x[l + 1], (double)cv.y);
            dist = __dadd_rn(dist, __dmul_rn(diff, diff));
            diff = __dsub_rn((double)x[l + 2], (double)cv.z);
            dist = __dadd_rn(dist, __dmul_rn(diff, diff));
            diff = __dsub_rn((double)x[l + 3], (double)cv.w);
            dist = __dadd_rn(dist, __dmul_rn(diff, diff));
        }
        if (dist < best) { best = dist; arg = j; }
    }
    // smallest distance of the wave, then the smallest index among the lanes that hold it
    const double wbest = wave_min_f64(best);
    const unsigned long long tied = __ballot(best == wbest);
    // up to 64 centroids a lane's index is its number: the first lane that holds the minimum has the smallest index
    if (k <= 64) return __ffsll((long long)tied) - 1;
    return wave_min_i32(best == wbest ? arg : 0x7fffffff);
}

// v = h + m + l exactly, each piece a bf16 (8 significant bits): h and m by truncation, l is what is left
__device__ inline void split3(float v, unsigned &h, unsigned &m, unsigned &l)
{
    const unsigned b = __float_as_uint(v);
    h = b >> 16;
    const float r = v - __uint_as_float(b & 0xffff0000u);
    const unsigned rb = __float_as_uint(r);
    m = rb >> 16;
    const float r2 = r - __uint_as_float(rb & 0xffff0000u);
    l = __float_as_uint(r2) >> 16;
}

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }

// Two fp16 pieces of a value, rounded toward zero: v = h + l + r with |r| < 2^-20 |v| while the pieces are normal
// fp16 numbers (11 significant bits each; v - h is exact in fp32).  The pair form packs a's pieces into the low
// halves and b's into the high halves, as two neighbouring operand elements.
typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
__device__ inline void split2_pair(float a, float b, unsigned &h, unsigned &l)
{
    const fp16x2 hh = __builtin_amdgcn_cvt_pkrtz(a, b);
    h = __builtin_bit_cast(unsigned, hh);
    const float ra = a - (float)hh[0], rb = b - (float)hh[1];
    l = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(ra, rb));
}
__device__ inline void split2(float v, unsigned short &h, unsigned short &l)
{
    unsigned ph, pl;
    split2_pair(v, 0.0f, ph, pl);
    h = (unsigned short)(ph & 0xffffu);
    l = (unsigned short)(pl & 0xffffu);
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

// (bits & mask) | idx.  The mask is kept opaque to the compiler (a VGPR) so that this selects one and-or
// instruction with the index as its scalar operand.  It must stay a compiler-visible operation (not inline
// assembly): it reads MFMA results, and the wait states between an MFMA and the first read of its result
// are inserted by the compiler.
__device__ inline int pack_key(float v, int mask, int idx)
{
    return (__float_as_int(v) & mask) | idx;
}

// median of three; the compiler selects the single med3 instruction for this shape
__device__ inline int med3i(int a, int b, int c) { return max(min(a, b), min(max(a, b), c)); }

// insert a key into the ascending pair (m1, m2) of the smallest keys seen so far
__device__ inline void insert2(int key, int &m1, int &m2)
{
    m2 = med3i(m1, m2, key);      // second smallest of {m1, m2, key} given m1 <= m2
    m1 = min(m1, key);
}

// insert two keys at once: the new smallest is the smallest of {m1, a, b} (one min3); the second smallest of
// {m1, m2, a, b} is the smaller of m2 and the second smallest of {m1, a, b} (one med3, one min), because m2 >= m1
__device__ inline void insert2x2(int a, int b, int &m1, int &m2)
{
    const int second = med3i(m1, a, b);
    // (written as one instruction: left to itself the compiler takes two minima here; the operands are packed keys,
    // results of vector instructions, so no wait states of the matrix pipeline are involved)
    asm("v_min3_i32 %0, %1, %2, %3" : "=v"(m1) : "v"(m1), "v"(a), "v"(b));
    m2 = min(m2, second);
}

// fold the 16 results of one 32x32 tile (4 quads of 4 rows) into the per-run states: the two smallest keys
// (five vector instructions per two distances: two and-or, min3, med3, min).  The second key shows whether the
// first is a clear winner.
template <int S, int ST>
__device__ inline void fold_tile(const floatx16 &acc, const int (&kidx)[16], int mask, int (&m1)[ST], int (&m2)[ST])
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int st = state_of<S>(q);
#pragma unroll
        for (int i = 0; i < 4; i += 2)
            insert2x2(pack_key(acc[4 * q + i], mask, kidx[4 * q + i]), pack_key(acc[4 * q + i + 1], mask, kidx[4 * q + i + 1]),
                      m1[st], m2[st]);
    }
}

// Everything a wave needs to run its share of a chunk.  The waves of a workgroup share the group's
// operand rows, centroid copy and integer accumulators (LDS), but each wave owns its points from the global
// load to the accumulator update, so there is no barrier inside the tile loop and waves in different phases
// (matrix pipeline / vector ALU / LDS atomics) overlap on a SIMD.
struct WaveCtx {
    const uint4 *opA_s;           // LDS: operand slots of the group's tiles
    const float *cs;              // LDS: the group's centroids as given, rows of DP + 4 floats, zero past feature d
    unsigned long long *sums;     // LDS: fixed-point sum deltas [copy][row][DP + 1]
    int *cnts;                    // LDS: member count deltas [copy][row]
    int copies, real_rows;        // accumulator copies (a power of two) and rows per copy
    const float *mu_s;            // LDS: -(column mean * scale) [32]
    float scale;                  // power of two that brings the centred data into fp16 range
    const int *shift_s;           // LDS: fixed-point shifts [32]
    const int *pow2hi_s;          // LDS: high words of the doubles 2^shift [32]
    const int *wide_s;            // LDS: wide-column flags [32], any at [32]
    const float *cnmax_s;         // LDS: per-run maximum squared norm of the centred centroids [8]
    const float *X;               // this space's rows
    const uint4 *xp;              // global: prepared copy of this space's points (see prep_block_u4_of)
    unsigned long long *log;      // global: this wave's ring of moved-pair records [kLogCap]
    int64_t ldx, N;
    int d, k0, n_runs, n_tiles, grow0;
    unsigned char *prev;          // global: labels of the last round for the group's run slots, [point][8 / S]
    int32_t *labels_out;          // global: labels of the group's runs [run][N] (final pass) or null
    long long *losum;             // global: low-order sums of wide columns [row][d]
    int64_t chunk_begin, chunk_end;
    int *next_slab;               // LDS: next slab of the chunk to hand out
    bool vec_x;                   // rows of X may be read 16 bytes at a time
    bool first_round;             // no point has a label yet
    float eps_a;
};

// VEC: rows of X may be read 16 bytes at a time.  A template parameter and not a run-time branch: with both load
// paths in one function the compiler merges them into 4-byte loads, and a wave's rows then cost four times the
// cache look-ups (which bounds sweeps over few k).
// PRE: the operands come from the prepared copy; the raw rows are read on demand (not in a pass that sums the loss,
// which needs every row, and not in the first round, where every row enters a cluster).
template <int DP, int S, bool FINAL, bool TRACE, bool VEC, bool PRE>
__device__ inline void wave_loop(const WaveCtx &c, double (&jloc)[8])
{
    static_assert(!PRE || (!FINAL && !TRACE), "the prepared copy serves the plain assign + update pass only");
    constexpr int NB = slab_blocks_of(DP, S);       // blocks of 32 points per wave and slab
    // with 2 blocks at d_pad = 32 the rows of the next slab are requested after the tile loop, when the operand
    // registers are free again, instead of before it
    constexpr bool LATE_FETCH = DP == 32 && NB == 2;
    constexpr int H = DP / 2;                       // features per half-wave
    constexpr int CS = DP + 4;                      // row stride of the LDS copy of the centroids
    constexpr int NK = ksteps_of(DP);               // K-steps of 16 per cross term
    constexpr int NS = tile_slots_of(DP);           // operand slots per tile and lane
    constexpr int HP = 8 * NK;                      // feature slots per half-wave (H padded to whole K-steps)
    constexpr int ST = S == 1 ? 4 : (S == 2 ? 2 : 1);   // runs owned by a lane
    constexpr int SLAB_ = 32 * NB;                  // points a wave takes at a time
    constexpr int NM = 3 * NK + 1;                  // MFMAs per tile block
    constexpr int VPER = (40 + 16 + NM - 1) / NM;   // vector ops to slot in after each MFMA of a chain
    constexpr bool LOSS = FINAL || TRACE;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hl = lane >> 5;
    const int d = c.d;
    const int f0 = hl * H;                          // first feature of this lane's half
    const int nf = min(max(d - f0, 0), H);          // real features of this lane's half
    const uint4 *opA_s = c.opA_s;
    int mask = (int)0xffffff80;
    asm volatile("" : "+v"(mask));                  // keep the mask in a VGPR

    const bool any_wide = c.wide_s[32] != 0;
    // this lane's copy of the accumulators
    unsigned long long *const sums_l = c.sums + (lane & (c.copies - 1)) * c.real_rows * (DP + 1);
    int *const cnts_l = c.cnts + (lane & (c.copies - 1)) * c.real_rows;

    // Raw features of this lane's half of its points.  The rows of the next step are loaded while this step
    // runs: the loads are unconditional (addresses clamped into the chunk and the row, masking happens when the
    // values are used) and nothing touches their registers before settle(), so no wait is placed early.
    // Addresses are a wave-uniform base (the slab's first row) plus a 32-bit lane offset: the row index inside
    // the slab is clamped to the chunk's last row, the feature offset to the row's last 16 bytes.
    float xnext[PRE ? 1 : NB][PRE ? 1 : HP];
    constexpr int NP = prep_slots_of(DP);            // operand slots per lane and block in the prepared copy
    uint4 pnext[PRE ? NB : 1][PRE ? NP : 1];          // PRE: the operand slots of the slab being fetched
    uint2 nnext[PRE ? NB : 1];                        // PRE: its norm entries
    const unsigned ldx32 = (unsigned)c.ldx;          // checked on the host: 64 rows of ldx floats fit 32 bits
    // this lane's clamped feature offsets (fixed for the launch; with the prepared copy they are worked out where
    // a row is read, which is rare, instead of being kept in registers)
    auto feat_off = [&](int s) { return (unsigned)(VEC ? min(f0 + (s & ~3), d - 4) + (s & 3) : min(f0 + s, d - 1)); };
    unsigned foff[PRE ? 1 : H];
    if constexpr (!PRE) {
#pragma unroll
        for (int s = 0; s < H; ++s) foff[s] = feat_off(s);
    }
    // The labels of the last round are kept per group as one byte per (point, run slot of the group), the R = 8 / S
    // slots of a point side by side: a lane reads and writes the labels of its ST runs as one word.
    constexpr int R = 8 / S;                         // run slots of the group
    using LabWord = std::conditional_t<ST == 4, unsigned, std::conditional_t<ST == 2, unsigned short, unsigned char>>;
    const unsigned lab_off = S == 8 ? 0u : (unsigned)(hl * ST);     // this lane's first byte within a point's R bytes
    unsigned oldn[NB];                               // previous labels of the slab being fetched (byte st: run st of this lane)
    unsigned run_off[ST];                            // offset of this lane's runs in the label output (runs are N apart)
    unsigned actmask = 0u;                           // bytes of a label word that belong to real runs of this lane
#pragma unroll
    for (int st = 0; st < ST; ++st) {
        const unsigned rl = S == 8 ? 0u : (unsigned)(hl * ST + st);
        run_off[st] = min(rl, (unsigned)(c.n_runs - 1)) * (unsigned)c.N;
        if (((S == 8) ? (hl == 0) : true) && (int)rl < c.n_runs) actmask |= 0xffu << (8 * st);
    }
    for (int pb = 0; pb < NB; ++pb) oldn[pb] = 0xffffffffu;
    unsigned char *const prev_chunk = c.prev + c.chunk_begin * R;          // the chunk's first label byte
    const unsigned chunk_pts = (unsigned)(c.chunk_end - c.chunk_begin);   // points of the chunk (at most 2^17)
    auto load_labels = [&](int64_t slab_base, unsigned li) -> unsigned {
        const unsigned pt = (unsigned)(slab_base - c.chunk_begin) + li;   // point within the chunk
        return (unsigned)*reinterpret_cast<const LabWord *>(prev_chunk + (pt * (unsigned)R + lab_off));
    };
    auto fetch = [&](int64_t slab_base) {
        const float *Xs = c.X + slab_base * c.ldx;
        const unsigned last = (unsigned)min((int64_t)(SLAB_ - 1), c.chunk_end - 1 - slab_base);
        if constexpr (PRE) {
            const int64_t blk0 = slab_base >> 5, blk_last = (c.chunk_end - 1) >> 5;     // chunks start on a block boundary
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
                const uint4 *bp = c.xp + min(blk0 + pb, blk_last) * prep_block_u4_of(DP);
#pragma unroll
                for (int sl = 0; sl < NP; ++sl) pnext[pb][sl] = bp[sl * 64 + lane];
                nnext[pb] = reinterpret_cast<const uint2 *>(bp + NP * 64)[n];
                const unsigned li = min((unsigned)(pb * 32 + n), last);
                oldn[pb] = load_labels(slab_base, li);
            }
            return;
        }
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            const unsigned li = min((unsigned)(pb * 32 + n), last);
            const unsigned ro = li * ldx32;
            if (VEC) {
#pragma unroll
                for (int c4 = 0; c4 < H / 4; ++c4) {
                    const float4 v = *reinterpret_cast<const float4 *>(Xs + (ro + foff[4 * c4]));
                    xnext[pb][4 * c4 + 0] = v.x; xnext[pb][4 * c4 + 1] = v.y; xnext[pb][4 * c4 + 2] = v.z; xnext[pb][4 * c4 + 3] = v.w;
                }
            } else {
#pragma unroll
                for (int s = 0; s < H; ++s) xnext[pb][s] = Xs[ro + foff[s]];
            }
            // labels these (point, run) pairs had in the previous round, 0xff before the first one
            if (!FINAL) oldn[pb] = load_labels(slab_base, li);
        }
    };
    // the outstanding loads of fetch() have to be complete here
    auto settle = [&]() {
        if constexpr (PRE) {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
#pragma unroll
                for (int sl = 0; sl < NP; ++sl)
                    asm volatile("" : "+v"(pnext[pb][sl].x), "+v"(pnext[pb][sl].y), "+v"(pnext[pb][sl].z), "+v"(pnext[pb][sl].w));
                asm volatile("" : "+v"(nnext[pb].x), "+v"(nnext[pb].y));
            }
        } else {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                for (int s = 0; s < H; ++s) asm volatile("" : "+v"(xnext[pb][s]));
        }
        if (!FINAL) {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) asm volatile("" : "+v"(oldn[pb]));
        }
    };
    // The chunk is handed out in slabs of SLAB points: one per wave statically, the rest from a counter in
    // LDS, so the waves of the workgroup finish together however their close calls and updates are spread.
    constexpr int SLAB = SLAB_;
    const int n_slabs = (int)((c.chunk_end - c.chunk_begin + SLAB - 1) / SLAB);
    // (a pass that sums the loss hands its slabs out in a fixed order instead - wave w takes slabs w, w + waves, ... -
    // so that the fp64 partial sums of a wave, and with them the reported loss, are the same in every run)
    int fixed_next = wave;
    const int n_waves = (int)(blockDim.x >> 6);
    auto grab = [&]() -> int {
        if (LOSS) {
            fixed_next += n_waves;
            return fixed_next;
        }
        int v = 0;
        if (lane == 0) v = atomicAdd(c.next_slab, 1);
        return __builtin_amdgcn_readfirstlane(v);
    };
    // part of the error bound that belongs to a run (the centroids' largest squared norm), per run this lane owns
    float tol_run[ST];
#pragma unroll
    for (int st = 0; st < ST; ++st) tol_run[st] = c.eps_a * c.cnmax_s[S == 8 ? 0 : hl * ST + st] + kTolFloor;
    double jown[ST];                                 // loss sums of the runs this lane owns
#pragma unroll
    for (int st = 0; st < ST; ++st) jown[st] = 0.0;
    // ---- the log of moved pairs (PRE): records [log_head, log_tail) of the ring are waiting
    int log_head = 0, log_tail = 0;                  // wave-uniform
    auto log_flush = [&](int nrec) {
        // Works off `nrec` <= 64 records: a few lanes per record, eight features each (four at d_pad = 8) - the row is
        // read (16 bytes per load where rows can be read that way), put on the fixed-point grid and moved from the old
        // cluster's accumulators to the new one's.  Integer adds: the order in which records are worked off does not
        // matter.  What is the same for all lanes of a record (its fields, the row address, the accumulator rows) is
        // worked out by 4 (2, 2) lanes instead of one per feature, and a flush is 4 (2, 2) steps of 16 (32, 32) records.
        constexpr int FPL = DP >= 16 ? 8 : 4;   // features per lane
        constexpr int LPR = DP / FPL, RPS = 64 / LPR, STEPS = 64 / RPS, BATCH = STEPS < 4 ? STEPS : 4;   // steps whose rows are in flight together
        // The records were written by other lanes of this wave: their stores must have been issued to the memory
        // system before the reads.  Both go through this compute unit's own first-level cache, so workgroup scope is
        // enough (a wider scope would write back the second-level cache, which costs more than the whole flush).
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        unsigned long long rec = 0ull;
        if (lane < nrec) rec = __hip_atomic_load(&c.log[(unsigned)(log_head + lane) & (kLogCap - 1)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int fq = FPL * (lane % LPR), g = lane / LPR;     // this lane's first feature, its record within a step
        // this lane's feature columns in its copy of the accumulators (the lane group picks the copy)
        const int cp = g & (c.copies - 1);
        unsigned long long *const scol = c.sums + (int64_t)cp * c.real_rows * (DP + 1) + fq;
        const float *const xcol = c.X + c.chunk_begin * c.ldx + fq;
        // member counts: the lane that holds a record moves its one member, once per flush
        if (lane < nrec) {
            int *const ccol = c.cnts + (lane & (c.copies - 1)) * c.real_rows;
            const int nrow = (int)(((unsigned)rec >> 17) & 0xfffu), orow = (int)((unsigned)(rec >> 32) & 0xffffu);
            atomicAdd(ccol + nrow, 1);
            if (orow != 0xffff) atomicAdd(ccol + orow, -1);
        }
        int pow2hi[FPL];
#pragma unroll
        for (int j = 0; j < FPL; ++j) pow2hi[j] = c.pow2hi_s[fq + j];
        for (int s0 = 0; s0 < STEPS && s0 * RPS < nrec; s0 += BATCH) {
            unsigned lo[BATCH], hi[BATCH];
            float xv[BATCH][FPL];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int src = (s0 + u) * RPS + g;
                lo[u] = (unsigned)__shfl((int)(unsigned)rec, src, 64);
                hi[u] = (unsigned)__shfl((int)(unsigned)(rec >> 32), src, 64);
                const bool ok = src < nrec;
                const float *const row = xcol + (int64_t)(lo[u] & 0x1ffffu) * c.ldx;
                if (VEC) {
#pragma unroll
                    for (int h = 0; h < FPL / 4; ++h) {
                        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                        if (ok && fq + 4 * h < d) v = *reinterpret_cast<const float4 *>(row + 4 * h);     // d is a multiple of four here
                        xv[u][4 * h + 0] = v.x; xv[u][4 * h + 1] = v.y; xv[u][4 * h + 2] = v.z; xv[u][4 * h + 3] = v.w;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < FPL; ++j) xv[u][j] = (ok && fq + j < d) ? row[j] : 0.0f;
                }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int src = (s0 + u) * RPS + g;
                if (src < nrec) {
                    const int nrow = (int)((lo[u] >> 17) & 0xfffu), orow = (int)(hi[u] & 0xffffu);
                    unsigned long long *const srow_n = scol + nrow * (DP + 1);
                    unsigned long long *const srow_o = scol + orow * (DP + 1);
#pragma unroll
                    for (int j = 0; j < FPL; ++j) {
                        if (fq + j >= d) continue;
                        const unsigned long long v = any_wide ? (unsigned long long)to_fixed(xv[u][j], c.shift_s[fq + j]) + kFixBias
                                                              : fixed_biased(xv[u][j], pow2hi[j]);
                        atomicAdd(srow_n + j, v);
                        if (orow != 0xffff) __hip_atomic_fetch_sub(srow_o + j, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        if (any_wide && c.wide_s[fq + j] != 0) {
                            // bits below the grid of a wide column go to a global integer accumulator (rare)
                            const long long low = fixed_low(xv[u][j], c.shift_s[fq + j]);
                            if (low != 0) {
                                if (orow != 0xffff) atomicAdd(reinterpret_cast<unsigned long long *>(&c.losum[(int64_t)(c.grow0 + orow) * d + fq + j]), (unsigned long long)(-low));
                                atomicAdd(reinterpret_cast<unsigned long long *>(&c.losum[(int64_t)(c.grow0 + nrow) * d + fq + j]), (unsigned long long)low);
                            }
                        }
                    }
                }
            }
        }
        log_head += nrec;
    };
    int cur = wave;
    if (cur >= n_slabs) return;
    fetch(c.chunk_begin + (int64_t)cur * SLAB);
    settle();
    int nxt = grab();

    while (cur < n_slabs) {
        const int64_t base = c.chunk_begin + (int64_t)cur * SLAB;     // first point of this wave's slab
        // (a lane past the end of the chunk holds a copy of the chunk's last row: its pairs are never active)
        // (PRE: the raw rows are not there yet; the lanes that need theirs load them after the fold)
        float xraw[NB][HP];
        if constexpr (!PRE) {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
#pragma unroll
                for (int s = 0; s < HP; ++s) xraw[pb][s] = s < H ? xnext[pb][s] : 0.0f;
            }
        }
        if (!PRE && d < DP) {
            // padded features: the clamped loads brought real values of other features, they count as zero
#pragma unroll
            for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                for (int s = 0; s < H; ++s)
                    if (s >= nf) xraw[pb][s] = 0.0f;
        }
        const int nxt2 = grab();

        // ---- B operands of this lane's points: two fp16 pieces of the centred, scaled x' per K-step, and the bias
        // slot in bf16 (|x'|^2 in three pieces on the upper half-wave, ones on the lower: it meets (1,1,1 | pieces of |c'|^2))
        f16x8 bx[NB][2][NK];
        bf16x8 bb[NB];
        float xn[NB];
        int m1[NB][ST], m2[NB][ST];
        unsigned oldl[NB];                // labels in the previous round, one byte per run of this lane
        auto old_of = [&](int pb, int st) -> int { return (int)((oldl[pb] >> (8 * st)) & 0xffu); };
        if constexpr (PRE) {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) {
                    bx[pb][0][ks] = as_f16x8(pnext[pb][0 * NK + ks]);
                    bx[pb][1][ks] = as_f16x8(pnext[pb][1 * NK + ks]);
                }
                xn[pb] = (__uint_as_float(nnext[pb].x << 16) + __uint_as_float(nnext[pb].x & 0xffff0000u)) + __uint_as_float(nnext[pb].y << 16);
                bb[pb] = hl ? as_bf16x8(make_uint4(nnext[pb].x, nnext[pb].y, 0u, 0u)) : as_bf16x8(make_uint4(0x3f803f80u, 0x3f80u, 0u, 0u));
#pragma unroll
                for (int st = 0; st < ST; ++st) { m1[pb][st] = kBigKey; m2[pb][st] = kBigKey; }
                oldl[pb] = oldn[pb];
            }
        } else {
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            float xc[HP];
            float part = 0.0f;
#pragma unroll
            for (int s = 0; s < HP; ++s) {
                xc[s] = s < H ? fmaf(xraw[pb][s], c.scale, c.mu_s[f0 + s]) : 0.0f;   // (x - mean) * scale, one rounding
                part = fmaf(xc[s], xc[s], part);
            }
            xn[pb] = part + xchg32(part);
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) {
                unsigned ph[4], pl[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) split2_pair(xc[8 * ks + 2 * i], xc[8 * ks + 2 * i + 1], ph[i], pl[i]);
                bx[pb][0][ks] = as_f16x8(make_uint4(ph[0], ph[1], ph[2], ph[3]));
                bx[pb][1][ks] = as_f16x8(make_uint4(pl[0], pl[1], pl[2], pl[3]));
            }
            unsigned nh, nm, nl;
            split3(xn[pb], nh, nm, nl);
            bb[pb] = hl ? as_bf16x8(make_uint4(nh | (nm << 16), nl, 0u, 0u)) : as_bf16x8(make_uint4(0x3f803f80u, 0x3f80u, 0u, 0u));
#pragma unroll
            for (int st = 0; st < ST; ++st) { m1[pb][st] = kBigKey; m2[pb][st] = kBigKey; }
            oldl[pb] = oldn[pb];                    // fetched with the rows, a slab ago
        }
        }

        // The rows and previous labels of the next slab are asked for now and only needed when that slab starts, a
        // whole slab of work away.  Always issued - for the last slab it re-reads that slab - so that the number
        // of requests in flight is the same on every path.
        if (!LATE_FETCH) fetch(c.chunk_begin + (int64_t)min(nxt, n_slabs - 1) * SLAB);

        // ---- distances tile by tile; the results of one block are folded while the matrix pipeline runs the next
        // (the tile loop is written out twice so that the operand buffers and accumulators alternate by name
        // instead of being copied)
        uint4 a_even[NS], a_odd[NS];
        auto load_a = [&](uint4 (&dst)[NS], int t) {
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) dst[sl] = opA_s[(t * NS + sl) * 64 + lane];
        };
        load_a(a_even, 0);
        if constexpr (NB == 1) {
            // One block per slab: the four (d_pad = 32: seven) MFMAs of a tile form one dependent chain, so the wave interleaves them in
            // program order with the fold of the tile before - a quarter of the fold (one quad of rows) behind each MFMA -
            // and the two accumulators alternate by name.  The order is pinned: left to itself the compiler folds first
            // and then issues the chain into the same registers, and nothing of the wave overlaps.
            floatx16 acc_a, acc_b = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};     // (acc_b: never read before the second tile writes it)
            int kidx_prev[16];
            // `init`: the first tile of a slab - the first two keys of a run start its pair of smallest keys outright
            // (no sentinel values to set up and compare against)
            auto fold_quad = [&](const floatx16 &acc, const int (&kidx)[16], int q, auto init) {
                const int st = state_of<S>(q);
                const bool starts = decltype(init)::value && (S == 1 || (S == 2 && (q & 1) == 0) || (S >= 4 && q == 0));
                const int ka = pack_key(acc[4 * q], mask, kidx[4 * q]), kb = pack_key(acc[4 * q + 1], mask, kidx[4 * q + 1]);
                if (starts) {
                    m1[0][st] = min(ka, kb);
                    m2[0][st] = max(ka, kb);
                } else {
                    insert2x2(ka, kb, m1[0][st], m2[0][st]);
                }
                insert2x2(pack_key(acc[4 * q + 2], mask, kidx[4 * q + 2]), pack_key(acc[4 * q + 3], mask, kidx[4 * q + 3]),
                          m1[0][st], m2[0][st]);
            };
            // `fold`: 0 nothing to fold (first tile), 1 the tile before is the slab's first, 2 any later tile
            auto tile_step = [&](const uint4 (&a_cur)[NS], uint4 (&a_nxt)[NS], int t, auto fold, floatx16 &acc_new, const floatx16 &acc_old) {
                load_a(a_nxt, t + 1 < c.n_tiles ? t + 1 : t);
                int kidx[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    kidx[e] = key_index<S>(t, e >> 2, e & 3);
                    asm("" : "+s"(kidx[e]));
                }
                constexpr int kFold = decltype(fold)::value;
                using Init = std::integral_constant<bool, kFold == 1>;
                const floatx16 zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                // small cross terms first, then the leading one, then the bias slot: all in one fp32 accumulator; a quad of
                // the other accumulator is folded behind the last MFMA of each of the four parts
                acc_new = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[1 * NK]), bx[0][0][0], zero, 0, 0, 0);               // l.h
                if constexpr (NK == 2) acc_new = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[1 * NK + 1]), bx[0][0][1], acc_new, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (kFold) fold_quad(acc_old, kidx_prev, 0, Init{});
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) acc_new = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[ks]), bx[0][1][ks], acc_new, 0, 0, 0);   // h.l
                __builtin_amdgcn_sched_barrier(0);
                if (kFold) fold_quad(acc_old, kidx_prev, 1, Init{});
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) acc_new = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[ks]), bx[0][0][ks], acc_new, 0, 0, 0);   // h.h
                __builtin_amdgcn_sched_barrier(0);
                if (kFold) fold_quad(acc_old, kidx_prev, 2, Init{});
                __builtin_amdgcn_sched_barrier(0);
                acc_new = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_cur[2 * NK]), bb[0], acc_new, 0, 0, 0);                 // norms
                __builtin_amdgcn_sched_barrier(0);
                if (kFold) fold_quad(acc_old, kidx_prev, 3, Init{});
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 16; ++e) kidx_prev[e] = kidx[e];
            };
            using NoFold = std::integral_constant<int, 0>;
            using FoldFirst = std::integral_constant<int, 1>;
            using FoldLater = std::integral_constant<int, 2>;
            tile_step(a_even, a_odd, 0, NoFold{}, acc_a, acc_b);
            if (c.n_tiles == 1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) fold_quad(acc_a, kidx_prev, q, std::true_type{});
            } else {
                tile_step(a_odd, a_even, 1, FoldFirst{}, acc_b, acc_a);
                int t = 2;
                for (; t + 2 <= c.n_tiles; t += 2) {
                    tile_step(a_even, a_odd, t, FoldLater{}, acc_a, acc_b);
                    tile_step(a_odd, a_even, t + 1, FoldLater{}, acc_b, acc_a);
                }
                if (t < c.n_tiles) {
                    tile_step(a_even, a_odd, t, FoldLater{}, acc_a, acc_b);
                    fold_tile<S, ST>(acc_a, kidx_prev, mask, m1[0], m2[0]);
                } else {
                    fold_tile<S, ST>(acc_b, kidx_prev, mask, m1[0], m2[0]);
                }
            }
        } else {
        floatx16 acc_prev;                 // results of the block before the current one, folded one block late
            int kidx_old[16];
            // `first`: the very first block of the slab has no block before it to fold
            auto tile_step = [&](const uint4 (&a_cur)[NS], uint4 (&a_nxt)[NS], int t, auto first) {
                load_a(a_nxt, t + 1 < c.n_tiles ? t + 1 : t);
                // per-row key indices of this tile as opaque scalars (one scalar operand per and-or)
                int kidx[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    kidx[e] = key_index<S>(t, e >> 2, e & 3);
                    asm("" : "+s"(kidx[e]));
                }
#pragma unroll
                for (int pb = 0; pb < NB; ++pb) {
                    // small cross terms first, then the leading one, then the bias slot: all in one fp32 accumulator
                    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[1 * NK + ks]), bx[pb][0][ks], acc, 0, 0, 0);   // l.h
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[0 * NK + ks]), bx[pb][1][ks], acc, 0, 0, 0);   // h.l
#pragma unroll
                    for (int ks = 0; ks < NK; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a_cur[0 * NK + ks]), bx[pb][0][ks], acc, 0, 0, 0);   // h.h
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a_cur[2 * NK]), bb[pb], acc, 0, 0, 0);                                         // norms
                    if (pb == 0) {
                        if (!decltype(first)::value) fold_tile<S, ST>(acc_prev, kidx_old, mask, m1[NB - 1], m2[NB - 1]);
                    } else {
                        fold_tile<S, ST>(acc_prev, kidx, mask, m1[pb - 1], m2[pb - 1]);
                    }
#pragma unroll
                    for (int s = 0; s < NM; ++s) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x002, VPER, 0);   // then a share of the fold
                    }
                    acc_prev = acc;
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) kidx_old[e] = kidx[e];
            };
            {
                tile_step(a_even, a_odd, 0, std::true_type{});
                int t = 1;
                for (; t + 2 <= c.n_tiles; t += 2) {
                    tile_step(a_odd, a_even, t, std::false_type{});
                    tile_step(a_even, a_odd, t + 1, std::false_type{});
                }
                if (t < c.n_tiles) tile_step(a_odd, a_even, t, std::false_type{});
            }
            fold_tile<S, ST>(acc_prev, kidx_old, mask, m1[NB - 1], m2[NB - 1]);
        }
        if (LATE_FETCH) fetch(c.chunk_begin + (int64_t)min(nxt, n_slabs - 1) * SLAB);

        // ---- labels, close calls, sums
        constexpr int NBST = NB * ST;               // (block, run) pairs a lane owns
        // this lane's points within the chunk, and whether they exist (the last slab of a chunk may be ragged)
        const unsigned pt0 = (unsigned)(base - c.chunk_begin);
        unsigned ptl[NB];
        bool pvalid[NB];
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            ptl[pb] = pt0 + (unsigned)(pb * 32 + n);
            pvalid[pb] = ptl[pb] < chunk_pts;
        }
        // Keys: which pairs does the exact arithmetic have to confirm?  Bit pb * ST + st of a lane's mask, put together
        // only when the wave has such a pair at all.
        unsigned pend = 0;
        bool closeb[NB][ST];
        bool any_close = false;
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            if (S == 8) {
                // the run spans both half-waves: add the half bit to the index, then merge with the partner lane
                int k1 = m1[pb][0], k2 = m2[pb][0];
                if (k1 < kBigKey) k1 |= hl << 4;
                if (k2 < kBigKey) k2 |= hl << 4;
                const int o1 = xchg32(k1), o2 = xchg32(k2);
                insert2(o1, k1, k2);
                insert2(o2, k1, k2);
                m1[pb][0] = k1; m2[pb][0] = k2;
            }
#pragma unroll
            for (int st = 0; st < ST; ++st) {
                const int rl = S == 8 ? 0 : hl * ST + st;     // run within the group
                const bool active = ((S == 8) ? (hl == 0) : true) && rl < c.n_runs && pvalid[pb];
                // Error bound of the two expansions (rounding of norms, products and the centring) plus the 7
                // mantissa bits given up to the index.  The keys are compared as they are, index bits included:
                // read as a float a key g lies within 2^-16 |v| of the value v it was packed from, so
                // v2 - v1 >= g2 (1 - 2^-15) - g1 whenever g2 >= |g1| - and a negative g1 (a distance of zero
                // within the bound) is smaller than the bound's own slack.  One multiply-add and one compare.
                const float g1 = __int_as_float(m1[pb][st]), g2 = __int_as_float(m2[pb][st]);
                const float tol0 = fmaf(c.eps_a, xn[pb], tol_run[st]);
                closeb[pb][st] = active && !(fmaf(g2, 0.999969482421875f, -g1) > tol0);
                any_close = any_close || closeb[pb][st];
            }
        }
        if (__ballot(any_close) != 0ull) {
#pragma unroll
            for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                for (int st = 0; st < ST; ++st) pend |= (unsigned)closeb[pb][st] << (pb * ST + st);
        }

        // A close call (about one pair in a thousand on knob data; every pair where centroids coincide or integer
        // data ties exactly) is settled by the whole wave with the exact arithmetic over the run.  The point's row is
        // read out of the registers of the two lanes that hold its halves.
        auto settle_close_calls = [&](const float (&xr)[NB][HP]) {
            unsigned long long todo = __ballot(pend != 0u);
            while (todo) {
                const int src = __ffsll((long long)todo) - 1;
                const unsigned sbits = (unsigned)__builtin_amdgcn_readlane((int)pend, src);
                const int idx = __ffs(sbits) - 1, pb = idx / ST, st = idx % ST;
                const int srl = S == 8 ? 0 : (src >> 5) * ST + st;
                const float *crun = c.cs + (srl * c.k0 + srl * (srl - 1) / 2) * CS;
                float xs[DP];
#pragma unroll
                for (int s = 0; s < H; ++s) {
                    float v = xr[0][s];
#pragma unroll
                    for (int q = 1; q < NB; ++q)
                        if (pb == q) v = xr[q][s];
                    xs[s] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src & 31));
                    xs[H + s] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), (src & 31) + 32));
                }
                const int arg = exact_argmin_wave<DP>(xs, crun, CS, c.k0 + srl);
                if (lane == src) {
                    pend &= pend - 1u;
#pragma unroll
                    for (int i = 0; i < NBST; ++i)
                        if (i == idx) m1[i / ST][i % ST] = arg;
                }
                todo = __ballot(pend != 0u);
            }
        };
        if constexpr (PRE) {
            // Raw rows on demand: the exact arithmetic of a close call needs the point's row; both lanes of such a
            // point (each holds half of the features) load their half.  (The exact sums need the rows of the points
            // whose label changed: those are read when the wave works off its log of moved pairs.)  Loads, wait and
            // scans sit in one branch, so that a slab without close calls never waits on the memory counter here: what
            // is in flight then are the operands of the next slab, wanted a whole slab later.
            if (__ballot(pend != 0u) != 0ull) {
                unsigned need = pend;
                need |= xchg32(need);
                float xr[NB][HP];
#pragma unroll
                for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                    for (int s = 0; s < HP; ++s) xr[pb][s] = 0.0f;
                const float *Xs = c.X + base * c.ldx;
                // (the row index is made opaque here so that the offsets below are worked out on the spot: hoisted out
                // of the slab loop they would sit in registers, or in spill slots, through the tile loop)
                unsigned nrow = (unsigned)n;
                asm volatile("" : "+v"(nrow));
#pragma unroll
                for (int pb = 0; pb < NB; ++pb) {
                    if ((need >> (pb * ST)) & ((1u << ST) - 1u)) {       // an active pair: the point lies inside the chunk
                        const unsigned ro = ((unsigned)(pb * 32) + nrow) * ldx32;
                        if (VEC) {
#pragma unroll
                            for (int c4 = 0; c4 < H / 4; ++c4) {
                                const float4 v = *reinterpret_cast<const float4 *>(Xs + (ro + feat_off(4 * c4)));
                                xr[pb][4 * c4 + 0] = v.x; xr[pb][4 * c4 + 1] = v.y; xr[pb][4 * c4 + 2] = v.z; xr[pb][4 * c4 + 3] = v.w;
                            }
                        } else {
#pragma unroll
                            for (int s = 0; s < H; ++s) xr[pb][s] = Xs[ro + feat_off(s)];
                        }
                        if (d < DP) {
#pragma unroll
                            for (int s = 0; s < H; ++s)
                                if (s >= nf) xr[pb][s] = 0.0f;
                        }
                    }
                }
                // the rows have to be there before the branch ends (the wait belongs to this path alone)
#pragma unroll
                for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                    for (int s = 0; s < H; ++s) asm volatile("" : "+v"(xr[pb][s]));
                settle_close_calls(xr);
            }
        } else {
            settle_close_calls(xraw);
        }

        // labels are final: the new label word of every block, and which of its bytes differ from the last round's
        // (the stores wait until the end of the slab)
        unsigned neww[NB], diffw[NB];
        unsigned mv = 0;                            // bit pb * ST + st: that pair moved
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            // the low bytes of the keys side by side (byte permutes), index bits only
            unsigned w;
            if constexpr (ST == 4) {
                w = (__builtin_amdgcn_perm((unsigned)m1[pb][1], (unsigned)m1[pb][0], 0x0c0c0400u) |
                     __builtin_amdgcn_perm((unsigned)m1[pb][3], (unsigned)m1[pb][2], 0x04000c0cu)) & 0x7f7f7f7fu;
            } else if constexpr (ST == 2) {
                w = __builtin_amdgcn_perm((unsigned)m1[pb][1], (unsigned)m1[pb][0], 0x0c0c0400u) & 0x7f7fu;
            } else {
                w = (unsigned)m1[pb][0] & 127u;
            }
            neww[pb] = w;
            diffw[pb] = 0u;
            if (!FINAL) diffw[pb] = pvalid[pb] ? ((w ^ oldl[pb]) & actmask) : 0u;
        }
        if (!FINAL) {
            bool any = false;
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) any = any || diffw[pb] != 0u;
            if (__ballot(any) != 0ull) {
#pragma unroll
                for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                    for (int st = 0; st < ST; ++st) mv |= (unsigned)(((diffw[pb] >> (8 * st)) & 0xffu) != 0u) << (pb * ST + st);
            }
        }

        if constexpr (PRE) {
            // Exact sums, later: the moved pairs go into this wave's log; 64 records at a time are worked off below.
            static_assert(64 * NBST + 63 <= kLogCap, "a slab's records and what an earlier flush left over must fit the ring");
#pragma unroll
            for (int i = 0; i < NBST; ++i) {
                const bool has = (mv >> i) & 1u;
                const unsigned long long bal = __ballot(has);
                if (bal != 0ull) {
                    const int pb = i / ST, st = i % ST;
                    const unsigned rl = S == 8 ? 0u : (unsigned)(hl * ST + st);
                    const unsigned pos = (unsigned)log_tail +
                                         __builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
                    if (has) {
                        // the record names the point and the two accumulator rows (within the group) outright, so
                        // that working it off takes no arithmetic on runs and labels
                        const unsigned pt = ptl[pb];                                                       // below 2^17
                        const unsigned rowbase = rl * (unsigned)c.k0 + rl * (rl - 1u) / 2u;
                        const unsigned lo = pt | ((rowbase + (unsigned)(m1[pb][st] & 127)) << 17);         // rows: below 2^12
                        const unsigned hi = old_of(pb, st) == 0xff ? 0xffffu : rowbase + (unsigned)old_of(pb, st);
                        c.log[pos & (kLogCap - 1)] = ((unsigned long long)hi << 32) | lo;
                    }
                    log_tail += (int)__popcll(bal);
                }
            }
            while (log_tail - log_head >= 64) log_flush(64);
        }
        if (!FINAL && !PRE) {
            // Exact sums: a point whose label changed moves its fixed-point row from the old cluster to the new
            // one.  Both lanes of the point's pair take part (each holds half of the features); one pair per pass.
            const unsigned mvo = xchg32(mv);
            unsigned both = hl ? (mvo | (mv << NBST)) : (mv | (mvo << NBST));
            // bits below the grid of a wide column go to a global integer accumulator (rare)
            auto add_low = [&](int64_t p, int rowbase, int ol, int nl) {
                const int64_t crow = c.grow0 + rowbase;
                for (int s = 0; s < nf; ++s) {
                    if (c.wide_s[f0 + s] == 0) continue;
                    const long long lo = fixed_low(c.X[p * c.ldx + f0 + s], c.shift_s[f0 + s]);
                    if (lo == 0) continue;
                    if (ol != 0xff) atomicAdd(reinterpret_cast<unsigned long long *>(&c.losum[(crow + ol) * d + f0 + s]), (unsigned long long)(-lo));
                    atomicAdd(reinterpret_cast<unsigned long long *>(&c.losum[(crow + nl) * d + f0 + s]), (unsigned long long)lo);
                }
            };
            if (__ballot(both != 0u) != 0ull) {
                // this lane's half of its points' rows on the fixed-point grid (zero beyond the last feature)
                unsigned long long fx[NB][H];
                if (any_wide) {
                    // some column has bits below its grid: those are cut off here (and summed apart, see add_low)
#pragma unroll
                    for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                        for (int s = 0; s < H; ++s) fx[pb][s] = (unsigned long long)to_fixed(xraw[pb][s], c.shift_s[f0 + s]) + kFixBias;
                } else {
#pragma unroll
                    for (int pb = 0; pb < NB; ++pb)
#pragma unroll
                        for (int s = 0; s < H; ++s) fx[pb][s] = fixed_biased(xraw[pb][s], c.pow2hi_s[f0 + s]);   // xraw is 0 past the last feature
                }
                if (c.first_round) {
                    // no point has a label yet: every pair of the slab enters its cluster, run by run
#pragma unroll
                    for (int pb = 0; pb < NB; ++pb) {
                        const int64_t p = base + pb * 32 + n;
                        for (int r = 0; r < c.n_runs; ++r) {
                            const int oh = S == 8 ? 0 : r / ST, ost = S == 8 ? 0 : r % ST;
                            int nl = 0;
#pragma unroll
                            for (int st = 0; st < ST; ++st)
                                if (st == ost) nl = m1[pb][st] & 127;
                            const int nlo = xchg32(nl);
                            if (hl != oh) nl = nlo;
                            const int rowbase = r * c.k0 + r * (r - 1) / 2;
                            if (pvalid[pb]) {
                                unsigned long long *sn = sums_l + (rowbase + nl) * (DP + 1) + f0;
#pragma unroll
                                for (int s = 0; s < H; ++s) atomicAdd(sn + s, fx[pb][s]);
                                if (hl == 0) atomicAdd(&cnts_l[rowbase + nl], 1);
                                if (any_wide) add_low(p, rowbase, 0xff, nl);
                            }
                        }
                    }
                } else do {
                    const bool act = both != 0u;
                    const int bit = act ? __ffs(both) - 1 : 0;
                    both &= both - 1u;
                    const int oh = bit / NBST, idx = bit % NBST, pb = idx / ST, st = idx % ST;
                    int kk = 0;                         // the owner's (old << 8) | new
#pragma unroll
                    for (int i = 0; i < NBST; ++i)
                        if (i == idx) kk = (m1[i / ST][i % ST] & 127) | (old_of(i / ST, i % ST) << 8);
                    const int kko = xchg32(kk);
                    if (hl != oh) kk = kko;
                    const int nl = kk & 0xff, ol = kk >> 8;
                    const int r = S == 8 ? 0 : oh * ST + st;
                    const int rowbase = r * c.k0 + r * (r - 1) / 2;
                    if (act) {
                        unsigned long long *sn = sums_l + (rowbase + nl) * (DP + 1) + f0;
                        unsigned long long v[H];
#pragma unroll
                        for (int s = 0; s < H; ++s) {
                            v[s] = fx[0][s];
#pragma unroll
                            for (int q = 1; q < NB; ++q)
                                if (pb == q) v[s] = fx[q][s];
                            atomicAdd(sn + s, v[s]);
                        }
                        if (hl == 0) atomicAdd(&cnts_l[rowbase + nl], 1);
                        if (ol != 0xff) {   // 0xff: no label yet, nothing to take back
                            unsigned long long *so = sums_l + (rowbase + ol) * (DP + 1) + f0;
#pragma unroll
                            for (int s = 0; s < H; ++s)
                                __hip_atomic_fetch_sub(so + s, v[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                            if (hl == 0) atomicAdd(&cnts_l[rowbase + ol], -1);
                        }
                        if (any_wide) add_low(base + pb * 32 + n, rowbase, ol, nl);
                    }
                } while (__ballot(both != 0u) != 0ull);
            }
        }
        if (LOSS) {
            // Loss of this assignment: every lane sums, for each (point, run) pair it owns, the exact squared distance
            // to the assigned centroid over all features in rising order; the other half of the row comes from the
            // partner lane by register swap.  Padded features are zero on both sides and add +0.
#pragma unroll
            for (int pb = 0; pb < NB; ++pb) {
                float xf[DP];
#pragma unroll
                for (int s = 0; s < H; ++s) {
                    const float other = xchg32(xraw[pb][s]);
                    xf[s] = hl ? other : xraw[pb][s];
                    xf[H + s] = hl ? xraw[pb][s] : other;
                }
#pragma unroll
                for (int st = 0; st < ST; ++st) {
                    const int rl = S == 8 ? 0 : hl * ST + st;
                    const bool active = ((S == 8) ? (hl == 0) : true) && rl < c.n_runs && pvalid[pb];
                    const int row = active ? rl * c.k0 + rl * (rl - 1) / 2 + (m1[pb][st] & 127) : 0;
                    const float *crow = c.cs + row * CS;
                    double dist = 0.0;
#pragma unroll
                    for (int l = 0; l < DP; l += 4) {
                        const float4 cv = *reinterpret_cast<const float4 *>(crow + l);
                        double diff = __dsub_rn((double)xf[l], (double)cv.x);
                        dist = __dadd_rn(dist, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xf[l + 1], (double)cv.y);
                        dist = __dadd_rn(dist, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xf[l + 2], (double)cv.z);
                        dist = __dadd_rn(dist, __dmul_rn(diff, diff));
                        diff = __dsub_rn((double)xf[l + 3], (double)cv.w);
                        dist = __dadd_rn(dist, __dmul_rn(diff, diff));
                    }
                    if (active) jown[st] = __dadd_rn(jown[st], dist);
                }
            }
        }
        // The rows of the next slab have to be there now.  Asking here, before this slab's stores are issued, keeps
        // the in-order memory counter from tying the next slab to those stores.
        settle();
#pragma unroll
        for (int pb = 0; pb < NB; ++pb) {
            const int64_t p = base + pb * 32 + n;
            if (FINAL) {
#pragma unroll
                for (int st = 0; st < ST; ++st) {
                    const int rl = S == 8 ? 0 : hl * ST + st;
                    const bool active = ((S == 8) ? (hl == 0) : true) && rl < c.n_runs && p < c.chunk_end;
                    const unsigned off = run_off[st] + (unsigned)(pb * 32 + n);      // used for active pairs only: inside the chunk
                    if (active && c.labels_out) (c.labels_out + base)[off] = m1[pb][st] & 127;
                }
            } else {
                // a word with a changed byte is written back whole (bytes of run slots without a run are never looked at)
                if (diffw[pb] != 0u) *reinterpret_cast<LabWord *>(prev_chunk + (ptl[pb] * (unsigned)R + lab_off)) = (LabWord)neww[pb];
            }
        }
        cur = nxt;
        nxt = nxt2;
    }
    if constexpr (PRE) {
        if (log_tail > log_head) log_flush(log_tail - log_head);
    }
    if (LOSS) {
        // hand the sums over by run: run r of the group is owned by half-wave r / ST (by the lower one when S = 8)
#pragma unroll
        for (int r = 0; r < 8 / S; ++r) {
            const int oh = S == 8 ? 0 : r / ST, ost = S == 8 ? 0 : r % ST;
            jloc[r] = hl == oh ? jown[ost] : 0.0;
        }
    }
}

template <int DP, bool FINAL, bool TRACE, bool VEC, bool PRE>
__device__ inline void wave_loop_of(int S, const WaveCtx &c, double (&jloc)[8])
{
    switch (S) {
    case 1: wave_loop<DP, 1, FINAL, TRACE, VEC, PRE>(c, jloc); break;
    case 2: wave_loop<DP, 2, FINAL, TRACE, VEC, PRE>(c, jloc); break;
    case 4: wave_loop<DP, 4, FINAL, TRACE, VEC, PRE>(c, jloc); break;
    default: wave_loop<DP, 8, FINAL, TRACE, VEC, PRE>(c, jloc); break;
    }
}

template <int DP, bool FINAL, bool TRACE, bool PRE>
__global__ void __launch_bounds__(step_threads_of(DP)) lloyd_step_kernel(SweepPlan plan, StepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int TH = step_threads_of(DP), WV = TH / 64;

    // Workgroup order: the chunks of all spaces of the batch, numbered space by space, are taken in blocks of
    // plan.chunk_block; within a block the groups go heaviest first (the dispatcher hands workgroups out in index order,
    // light ones fill the end), and the workgroups of all groups for one chunk sit a multiple of eight apart - they run
    // at about the same time on the same XCD, so that what one of them reads of the chunk (its rows or its part of the
    // prepared copy) the others find in that XCD's L2.
    int gi, chunk, b;
    {
        const int B = plan.chunk_block;
        const int n_all = plan.n_chunks * a.batch;          // chunks of the whole batch
        const int per_block = B * plan.n_groups;
        const int blk = blockIdx.x / per_block, rem = blockIdx.x % per_block;
        const int c0 = blk * B;
        const int bw = min(B, n_all - c0);                  // chunks of this block (the last one may be short)
        gi = plan.sched[rem / bw];
        const int vc = c0 + rem % bw;
        b = vc / plan.n_chunks;
        chunk = vc - b * plan.n_chunks;
        // The division leaves these in vector registers although they are the same in every lane.  At d_pad 32 the
        // kernel sits at the limit of 256 vector registers and spilled 35 of them over it (3% longer launches); as
        // scalars they cost none.
        b = __builtin_amdgcn_readfirstlane(b);
        chunk = __builtin_amdgcn_readfirstlane(chunk);
        gi = __builtin_amdgcn_readfirstlane(gi);
    }
    if (a.status[b] != 0) return;
    const GroupDesc g = plan.g[gi];
    const int d = a.d;
    const int k0 = plan.k_min + g.run0;                                   // k of the group's first run
    const int grow0 = rows_before(plan.k_min, g.run0);                    // first centroid row of the group
    const int real_rows = rows_before(plan.k_min, g.run0 + g.n_runs) - grow0;
    const int copies = g.copies;
    const Carve cv = carve_lds(DP, d, g.n_tiles, real_rows, copies);

    uint4 *opA_s = reinterpret_cast<uint4 *>(smem + cv.opA);
    float *cs_lds = reinterpret_cast<float *>(smem + cv.cs);
    unsigned long long *sums = reinterpret_cast<unsigned long long *>(smem + cv.sums);
    int *cnts = reinterpret_cast<int *>(smem + cv.cnts);
    float *mu_s = reinterpret_cast<float *>(smem + cv.misc);              // [32]
    int *shift_s = reinterpret_cast<int *>(smem + cv.misc + 128);         // [32]
    int *wide_s = reinterpret_cast<int *>(smem + cv.misc + 256);          // [32] + any at [32]
    float *cnmax_s = reinterpret_cast<float *>(smem + cv.misc + 400);     // [8]
    int *next_slab = reinterpret_cast<int *>(smem + cv.misc + 448);
    int *pow2hi_s = reinterpret_cast<int *>(smem + cv.misc + 1536);       // [32]
    double *jpart = reinterpret_cast<double *>(smem + cv.misc + 512);     // [8][WV]

    const int tid = threadIdx.x;
    char *wsb = a.ws + (int64_t)b * a.ws_bs;
    const float *Xb = a.X + (int64_t)b * a.x_bs;
    const float *Cb = a.C + (int64_t)b * a.c_bs;

    // group operands, centroids and column info into LDS; accumulators to zero
    {
        const float *colmean = reinterpret_cast<const float *>(wsb + a.off_colinfo);
        const int *colshift = reinterpret_cast<const int *>(wsb + a.off_colinfo + 128);
        const int *colwide = reinterpret_cast<const int *>(wsb + a.off_colinfo + 256);
        if (tid < 32) {
            mu_s[tid] = tid < DP ? colmean[tid] : 0.0f;                    // colmean: already negated and scaled
            shift_s[tid] = colshift[tid];
            pow2hi_s[tid] = (1023 + colshift[tid]) << 20;                 // 2^shift as a double: the high word
        }
        if (tid < 33) wide_s[tid] = colwide[tid];
        const uint4 *src = reinterpret_cast<const uint4 *>(wsb + a.off_opA + (int64_t)g.tile0 * tile_bytes_of(DP));
        for (int e = tid; e < g.n_tiles * (tile_bytes_of(DP) / 16); e += TH) opA_s[e] = src[e];
        {
            const float *csrc = Cb + (int64_t)grow0 * d;
            for (int e = tid; e < real_rows * DP; e += TH) {
                const int j = e / DP, l = e % DP;
                cs_lds[j * (DP + 4) + l] = l < d ? csrc[j * d + l] : 0.0f;
            }
        }
        if (tid == 0) *next_slab = WV;
        if (tid < 8) {
            // the largest squared norm of the run's centroids: the centroid kernel leaves one maximum per part of the run
            float m = 0.0f;
            if (tid < g.n_runs) {
                const float *parts = reinterpret_cast<const float *>(wsb + a.off_cnmax) + (g.run0 + tid) * kMaxParts;
                const int n_parts = (plan.k_min + g.run0 + tid + kPartRows - 1) / kPartRows;
                for (int p = 0; p < n_parts; ++p) m = fmaxf(m, parts[p]);
            }
            cnmax_s[tid] = m;
        }
        if (!FINAL) {
            for (int e = tid; e < copies * real_rows * (DP + 1); e += TH) sums[e] = 0ull;
            for (int e = tid; e < copies * real_rows; e += TH) cnts[e] = 0;
        }
    }
    __syncthreads();

    WaveCtx c;
    c.opA_s = opA_s;
    c.cs = cs_lds;            // the group's centroids as given, rows padded to d + 4 floats
    c.next_slab = next_slab;
    c.sums = sums; c.cnts = cnts; c.copies = copies; c.real_rows = real_rows; c.mu_s = mu_s; c.shift_s = shift_s; c.pow2hi_s = pow2hi_s; c.wide_s = wide_s; c.cnmax_s = cnmax_s;
    c.scale = *reinterpret_cast<const float *>(wsb + a.off_colinfo + kColScaleOff);
    c.xp = reinterpret_cast<const uint4 *>(wsb + a.off_xp);
    c.log = reinterpret_cast<unsigned long long *>(wsb + a.off_log) + ((int64_t)(gi * plan.n_chunks + chunk) * WV + (tid >> 6)) * kLogCap;
    c.X = Xb; c.ldx = a.ldx; c.N = a.N; c.d = d; c.k0 = k0; c.n_runs = g.n_runs; c.n_tiles = g.n_tiles; c.grow0 = grow0;
    c.prev = reinterpret_cast<unsigned char *>(wsb + a.off_prev) + (int64_t)g.lab0 * ((a.N + 15) / 16 * 16);
    c.labels_out = (FINAL && a.labels) ? a.labels + (int64_t)b * a.lab_bs + (int64_t)g.run0 * a.N : nullptr;
    c.losum = reinterpret_cast<long long *>(wsb + a.off_losum);
    c.chunk_begin = (int64_t)chunk * plan.chunk_len;
    c.chunk_end = min(a.N, c.chunk_begin + plan.chunk_len);
    // 16-byte loads need whole quads of features and aligned rows
    c.first_round = a.first_round != 0;
    c.vec_x = (d % 4 == 0) && (a.ldx % 4 == 0) && ((reinterpret_cast<uintptr_t>(Xb) & 15) == 0);
    // Bound on the summed error of two matrix-pipeline distances, relative to S = |x'|^2 + max |c'|^2 (centred and
    // scaled).  Per distance: what the two fp16 pieces per operand leave out - the product of the two low pieces and
    // the two remainders, each below 2^-20 of its element product - is at most 3 2^-20 |x'| |2c'| <= 24 2^-23 S; 4 or 7
    // chained MFMAs, each charged five fp32 roundings of a partial sum of at most 2 S (20 or 35 times 2^-23 S); fp32
    // norms d_pad 2^-24 S each; centring 2 2^-23 S: 54.5 2^-23 S at d_pad <= 16 and 77.5 2^-23 S at 32.  Twice that
    // is 109 and 155; the bound used is 120 and 200.  A piece below 2^-14 (an fp16 subnormal) is counted as lost
    // altogether: per distance at most 2^-14 sqrt(d) (|x'| + |2c'|) <= 2^-24 S + 0.078 d, hence the absolute term
    // kTolFloor next to the relative one (the 2^-24 S makes the 24 above 24.5).  (Measured on gfx950: one MFMA of this
    // shape is within 1.9 2^-24 of the sum of the magnitudes of its terms, against the five roundings charged.)
    c.eps_a = (float)(5 * ((DP < 16 ? 16 : DP) + 8)) * 1.1920928955078125e-07f;   // 5 (max(DP, 16) + 8) 2^-23

    double jloc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) jloc[i] = 0.0;

    if (c.chunk_begin < c.chunk_end) {
        if (c.vec_x) wave_loop_of<DP, FINAL, TRACE, true, PRE>(g.S, c, jloc);
        else wave_loop_of<DP, FINAL, TRACE, false, PRE>(g.S, c, jloc);
    }

    if (FINAL || TRACE) {
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            double v = jloc[i];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v = __dadd_rn(v, __shfl_xor(v, off, 64));
            if (lane == 0) jpart[i * WV + wave] = v;
        }
    }
    __syncthreads();   // every wave has finished its points: accumulators and partial losses are complete

    if (!FINAL) {
        unsigned long long *psum = reinterpret_cast<unsigned long long *>(wsb + a.off_psum) +
                                   ((int64_t)chunk * plan.total_rows + grow0) * d;
        for (int e = tid; e < real_rows * d; e += TH) {
            unsigned long long v = 0ull;
            long long rows_in = 0;     // rows that entered minus rows that left: each carried the bias once
            for (int cp = 0; cp < copies; ++cp) {
                v += sums[(cp * real_rows + e / d) * (DP + 1) + e % d];
                rows_in += cnts[cp * real_rows + e / d];
            }
            psum[e] = v - kFixBias * (unsigned long long)rows_in;
        }
        int *pcnt = reinterpret_cast<int *>(wsb + a.off_pcnt) + (int64_t)chunk * plan.total_rows + grow0;
        for (int e = tid; e < real_rows; e += TH) {
            int v = 0;
            for (int cp = 0; cp < copies; ++cp) v += cnts[cp * real_rows + e];
            pcnt[e] = v;
        }
    }
    if (FINAL || TRACE) {
        if (tid < g.n_runs) {
            double v = 0.0;
            for (int w = 0; w < WV; ++w) v = __dadd_rn(v, jpart[tid * WV + w]);
            reinterpret_cast<double *>(wsb + a.off_pj)[(int64_t)chunk * plan.n_runs + g.run0 + tid] = v;
        }
    }
}

// ---- column statistics: mean (for centring), fixed-point shift and range check ----------------
struct ColPart {
    double sum;
    int min_lsb, max_msb, bad, pad;
    float vmin, vmax;     // smallest and largest finite value
    int pad2[2];
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
    ColPart c = {0.0, 1 << 20, -(1 << 20), 0, 0, INFINITY, -INFINITY, {0, 0}};
    if (l < d) {
        // eight rows of this thread's column in flight at a time (the walk is bound by their latency); the values
        // are taken in row order, so the sum does not depend on the depth
        constexpr int U = 8;
        for (int64_t rb = r0 + pg; rb < r1; rb += (int64_t)U * ppp) {
            float xs[U];
#pragma unroll
            for (int u = 0; u < U; ++u) xs[u] = Xb[min(rb + (int64_t)u * ppp, r1 - 1) * ldx + l];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (rb + (int64_t)u * ppp >= r1) continue;
                const float x = xs[u];
                const unsigned bits = __float_as_uint(x);
                int e = (int)((bits >> 23) & 0xffu);
                unsigned m = bits & 0x7fffffu;
                if (e == 255) { c.bad = 1; continue; }
                c.sum = __dadd_rn(c.sum, (double)x);
                c.vmin = fminf(c.vmin, x);
                c.vmax = fmaxf(c.vmax, x);
                if (e == 0) { if (m == 0) continue; e = 1; } else m |= 0x800000u;
                const int lsb = e - 150 + (__ffs((int)m) - 1);
                const int msb = e - 150 + (31 - __clz((int)m));
                c.min_lsb = min(c.min_lsb, lsb);
                c.max_msb = max(c.max_msb, msb);
            }
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
            t.vmin = fminf(t.vmin, o.vmin);
            t.vmax = fmaxf(t.vmax, o.vmax);
        }
        reinterpret_cast<ColPart *>(ws + (int64_t)b * ws_bs + off_part)[blockIdx.x * 32 + tid] = t;
    }
}

__global__ void __launch_bounds__(256) colstats_final_kernel(int64_t N, int d, int n_blocks, char *ws, int64_t ws_bs, int64_t off_part,
                                                            int64_t off_colinfo, int32_t *status)
{
    // 256 threads: eight walk the partial results of one column, every eighth block each, eight loads in flight (the
    // walk is bound by their latency); the eight are then combined in a fixed order, so the mean is the same in every run
    constexpr int G = 8, U = 8;
    __shared__ int flags;
    __shared__ ColPart comb[G][32];
    const int b = blockIdx.x, l = threadIdx.x & 31, g = threadIdx.x >> 5;
    if (threadIdx.x == 0) flags = 0;
    const ColPart *part = reinterpret_cast<const ColPart *>(ws + (int64_t)b * ws_bs + off_part);
    ColPart t = {0.0, 1 << 20, -(1 << 20), 0, 0, INFINITY, -INFINITY, {0, 0}};
    if (l < d) {
        for (int g0 = g; g0 < n_blocks; g0 += G * U) {
            ColPart o[U];
#pragma unroll
            for (int u = 0; u < U; ++u) o[u] = part[min(g0 + u * G, n_blocks - 1) * 32 + l];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (g0 + u * G >= n_blocks) continue;
                t.sum = __dadd_rn(t.sum, o[u].sum);
                t.min_lsb = min(t.min_lsb, o[u].min_lsb);
                t.max_msb = max(t.max_msb, o[u].max_msb);
                t.bad |= o[u].bad;
                t.vmin = fminf(t.vmin, o[u].vmin);
                t.vmax = fmaxf(t.vmax, o[u].vmax);
            }
        }
    }
    comb[g][l] = t;
    __syncthreads();
    float mean = 0.0f;
    int shift = 0, wide = 0, msb = -(1 << 20);
    if (g == 0) {
        if (l < d) {
            for (int q = 1; q < G; ++q) {
                const ColPart o = comb[q][l];
                t.sum = __dadd_rn(t.sum, o.sum);
                t.min_lsb = min(t.min_lsb, o.min_lsb);
                t.max_msb = max(t.max_msb, o.max_msb);
                t.bad |= o.bad;
                t.vmin = fminf(t.vmin, o.vmin);
                t.vmax = fmaxf(t.vmax, o.vmax);
            }
            if (t.bad) atomicOr(&flags, RLS_STATUS_NONFINITE);
            else {
                mean = (float)(t.sum / (double)N);
                // largest distance of a value (or of a centroid, which lies between the extremes) from the mean; the
                // exponent of the next power of two above it, with the rounding of the two differences allowed for
                const float reach = fmaxf(t.vmax - mean, mean - t.vmin) * 1.000001f;
                if (reach > 0.0f) msb = ilogbf(reach);
                if (t.max_msb >= t.min_lsb) {
                    // grid: the finest bit kept by the main accumulator. |x * 2^shift| < 2^kGridBits, and a chunk moves
                    // at most 2^17 rows in and out of a cluster within 63 bits. Bits below the grid (wide columns) go to
                    // the low accumulator, which keeps kLowBits more; anything finer cannot be summed exactly.
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
        // One power of two for all columns (distances keep their order): with |x - mean| < 2^(M+1) in every column the
        // centred values obey |x - mean| * 2^(kScaledMsb - M - 2) < 2^(kScaledMsb - 1), one bit inside what fp16 holds for
        // 2 c'.  The exponent is kept inside the fp32 range; data that small only makes every comparison a close call.
        // (the 32 threads of the columns are the lower half of one wave: the exchange stays among them)
        for (int off = 16; off >= 1; off >>= 1) msb = max(msb, __shfl_xor(msb, off, 64));
        int e = kScaledMsb - 2 - (msb > -(1 << 20) ? msb : 0);
        e = min(max(e, -100), 100);
        const float scale = ldexpf(1.0f, e);
        colmean[l] = -(mean * scale);      // what the kernels add after multiplying by the scale
        colshift[l] = shift;
        colwide[l] = wide;
        if (l == 0) *reinterpret_cast<float *>(ws + (int64_t)b * ws_bs + off_colinfo + kColScaleOff) = scale;
        if (wide) atomicOr(&flags, 1 << 16);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int *colwide = reinterpret_cast<int *>(ws + (int64_t)b * ws_bs + off_colinfo + 256);
        colwide[32] = (flags >> 16) & 1;
        status[b] = flags & 0xffff;
    }
}

// ---- the prepared copy of the points (see prep_block_u4_of): what the step kernel would derive from a row in every
//      launch and for every group of runs - centring, scaling, the two fp16 pieces, the squared norm - done once per sweep.
//      One thread per (point, half of the features), in the lane order of the step kernel; the arithmetic is the
//      step kernel's own, instruction for instruction.
template <int DP>
__global__ void __launch_bounds__(256) lloyd_prepare_kernel(const float *__restrict__ X, int64_t N, int d, int64_t ldx, int64_t x_bs,
                                                            const int32_t *__restrict__ status, char *ws, int64_t ws_bs,
                                                            int64_t off_colinfo, int64_t off_xp)
{
    constexpr int H = DP / 2, NK = ksteps_of(DP), HP = 8 * NK;
    const int b = blockIdx.y;
    if (status[b] != 0) return;
    char *wsb = ws + (int64_t)b * ws_bs;
    const float *Xb = X + (int64_t)b * x_bs;
    const float *colmean = reinterpret_cast<const float *>(wsb + off_colinfo);      // -(mean * scale)
    const float scale = *reinterpret_cast<const float *>(wsb + off_colinfo + kColScaleOff);
    uint4 *xp = reinterpret_cast<uint4 *>(wsb + off_xp);
    const int64_t n_blocks = (N + 31) / 32;
    const int lane = threadIdx.x & 63, n = lane & 31, hl = lane >> 5;
    const int f0 = hl * H;
    for (int64_t blk = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); blk < n_blocks;
         blk += (int64_t)gridDim.x * (blockDim.x >> 6)) {
        const int64_t p = blk * 32 + n;
        float xc[HP];
        float part = 0.0f;
#pragma unroll
        for (int s = 0; s < HP; ++s) {
            const int f = f0 + s;
            const float x = (s < H && f < d && p < N) ? Xb[p * ldx + f] : 0.0f;
            // a point past the end and a padded feature count as a zero of the centred data
            xc[s] = (s < H && f < d && p < N) ? fmaf(x, scale, colmean[f]) : 0.0f;
            part = fmaf(xc[s], xc[s], part);
        }
        const float xn = part + xchg32(part);
        uint4 *bp = xp + blk * prep_block_u4_of(DP);
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            unsigned ph[4], pl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) split2_pair(xc[8 * ks + 2 * i], xc[8 * ks + 2 * i + 1], ph[i], pl[i]);
            bp[(0 * NK + ks) * 64 + lane] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
            bp[(1 * NK + ks) * 64 + lane] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
        }
        if (hl == 0) {
            unsigned nh, nm, nl;
            split3(xn, nh, nm, nl);
            reinterpret_cast<uint2 *>(bp + prep_slots_of(DP) * 64)[n] = make_uint2(nh | (nm << 16), nl);
        }
    }
}

// ---- start of a sweep: padding operand rows are zero vectors with a huge norm; running totals are zero;
//      no point has a label yet
struct InitArgs {
    char *ws;
    int64_t ws_bs;
    int64_t off_opA, off_losum, off_tot, off_totcnt, off_prev;
    int64_t n_tiles, n_losum, n_tot, n_totcnt, n_prev16;   // element counts (prev in 16-byte units)
    int32_t dp;
};
__global__ void sweep_init_kernel(InitArgs a)
{
    char *wsb = a.ws + (int64_t)blockIdx.y * a.ws_bs;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, step = (int64_t)gridDim.x * blockDim.x;
    uint4 *opA = reinterpret_cast<uint4 *>(wsb + a.off_opA);
    long long *losum = reinterpret_cast<long long *>(wsb + a.off_losum);
    long long *tot = reinterpret_cast<long long *>(wsb + a.off_tot);
    long long *totcnt = reinterpret_cast<long long *>(wsb + a.off_totcnt);
    uint4 *prev = reinterpret_cast<uint4 *>(wsb + a.off_prev);
    {
        // a row without a centroid: zero pieces and, in the bias slot, the pieces of a huge squared norm
        // (lower half-wave) next to the ones that meet the pieces of |x'|^2 (upper half-wave)
        const int ns = tile_slots_of(a.dp);
        unsigned ph, pm, pl;
        split3(kPadNorm, ph, pm, pl);
        for (int64_t e = t0; e < a.n_tiles * ns * 64; e += step) {
            const int sl = (int)((e / 64) % ns), ln = (int)(e % 64);
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (sl == ns - 1) v = ln < 32 ? make_uint4(ph | (pm << 16), pl, 0u, 0u) : make_uint4(0x3f803f80u, 0x3f80u, 0u, 0u);
            opA[e] = v;
        }
    }
    for (int64_t e = t0; e < a.n_losum; e += step) losum[e] = 0;
    for (int64_t e = t0; e < a.n_tot; e += step) tot[e] = 0;
    for (int64_t e = t0; e < a.n_totcnt; e += step) totcnt[e] = 0;
    const uint4 none = make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
    for (int64_t e = t0; e < a.n_prev16; e += step) prev[e] = none;
}

// Adds the per-chunk deltas of one (centroid, feature) element for chunks [c_begin, c_end) to a 128-bit sum and the
// member count deltas to cnt.  The values sit a whole chunk block apart in memory: eight loads are kept in flight,
// the walk is bound by their latency (integer sums: any order gives the same result).
__device__ inline void sum_chunks(const long long *pe, const int *pc, int64_t estride, int64_t cstride, int c_begin, int c_end,
                                  long long &hi, unsigned long long &lo, long long &cnt)
{
    constexpr int U = 8;
    int c0 = c_begin;
    for (; c0 + U <= c_end; c0 += U) {
        long long v[U];
        int m[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { v[u] = pe[(c0 + u) * estride]; m[u] = pc[(c0 + u) * cstride]; }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long nlo = lo + (unsigned long long)v[u];
            hi += (v[u] >> 63) + (nlo < lo ? 1 : 0);
            lo = nlo;
            cnt += m[u];
        }
    }
    for (; c0 < c_end; ++c0) {
        const long long v = pe[c0 * estride];
        const unsigned long long nlo = lo + (unsigned long long)v;
        hi += (v >> 63) + (nlo < lo ? 1 : 0);
        lo = nlo;
        cnt += pc[c0 * cstride];
    }
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
    int64_t off_colinfo, off_opA, off_cnmax, off_psum, off_pcnt, off_losum, off_tot, off_totcnt;
};

// One workgroup per run and part of kPartRows of its centroids: new centroids (from the seeding rows, or from the
// running totals after adding this round's per-chunk deltas), then the centred, -2-scaled MFMA operand rows and their
// squared norms.  (One workgroup per run left the large runs to the memory bandwidth of a single compute unit.)
template <int DP, bool INIT>
__global__ void __launch_bounds__(kThreads) lloyd_centroids_kernel(SweepPlan plan, CentroidArgs a)
{
    static_assert(kPartRows * DP <= kThreads, "one thread per (centroid, feature) element of a part");
    __shared__ float cs[kPartRows * DP];     // centred centroids of this part
    __shared__ long long part_hi[INIT ? 1 : kThreads], part_cnt[INIT ? 1 : kThreads];
    __shared__ unsigned long long part_lo[INIT ? 1 : kThreads];
    const int b = blockIdx.y, tid = threadIdx.x;
    if (a.status[b] != 0) return;
    // blockIdx.x counts the parts of all runs in run order: the run is the last one that starts at or before it
    const int parts0 = parts_upto(plan.k_min - 1);
    int run = 0;
    for (int step = 64; step >= 1; step >>= 1)
        if (run + step < plan.n_runs && parts_upto(plan.k_min + run + step - 1) - parts0 <= (int)blockIdx.x) run += step;
    const int d = a.d, k = plan.k_min + run;
    const int part = (int)blockIdx.x - (parts_upto(k - 1) - parts0);
    const int j0 = part * kPartRows, rows = min(kPartRows, k - j0);
    const int row0 = rows_before(plan.k_min, run);
    int gi = 0;
    while (gi + 1 < plan.n_groups && plan.g[gi + 1].run0 <= run) ++gi;
    const GroupDesc g = plan.g[gi];
    const int rl = run - g.run0;
    char *wsb = a.ws + (int64_t)b * a.ws_bs;
    const float *colmean = reinterpret_cast<const float *>(wsb + a.off_colinfo);   // -(mean * scale)
    const int *colshift = reinterpret_cast<const int *>(wsb + a.off_colinfo + 128);
    const int *colwide = reinterpret_cast<const int *>(wsb + a.off_colinfo + 256);
    const float scale = *reinterpret_cast<const float *>(wsb + a.off_colinfo + kColScaleOff);
    float *Cb = a.C + (int64_t)b * a.c_bs;
    // operand block of the group: per tile, tile_slots_of(DP) slots of 64 lanes x 8 halves (fp16 pieces, bf16 bias)
    unsigned short *opA = reinterpret_cast<unsigned short *>(wsb + a.off_opA + (int64_t)g.tile0 * tile_bytes_of(DP));
    constexpr int NK = ksteps_of(DP), NS = tile_slots_of(DP);

    // The chunks are split over `nsl` thread slices per (centroid, feature) element, so that the per-chunk deltas are
    // not read one after the other by a handful of threads; integer sums, any order.
    const int E = rows * DP;
    const int nsl = INIT ? 1 : kThreads / E;
    if (!INIT) {
        const int e = tid % E, sl = tid / E;
        const int j = j0 + e / DP, l = e % DP;
        long long hi = 0, cnt = 0;
        unsigned long long lo = 0;
        if (sl < nsl && l < d) {
            const long long *psum = reinterpret_cast<const long long *>(wsb + a.off_psum) + (int64_t)(row0 + j) * d + l;
            const int *pcnt = reinterpret_cast<const int *>(wsb + a.off_pcnt) + row0 + j;
            const int c_begin = (int)((int64_t)plan.n_chunks * sl / nsl), c_end = (int)((int64_t)plan.n_chunks * (sl + 1) / nsl);
            sum_chunks(psum, pcnt, (int64_t)plan.total_rows * d, plan.total_rows, c_begin, c_end, hi, lo, cnt);
        }
        part_hi[tid] = hi; part_lo[tid] = lo; part_cnt[tid] = cnt;
        __syncthreads();
    }

    if (tid < E) {
        const int e = tid;
        const int jj = e / DP, j = j0 + jj, l = e % DP;
        float cp = 0.0f;
        if (l < d) {
            float c;
            if (INIT) {
                const int64_t src = a.init_idx[(int64_t)b * a.init_bs + j];
                c = a.X[(int64_t)b * a.x_bs + src * a.ldx + l];
                Cb[(int64_t)(row0 + j) * d + l] = c;
            } else {
                long long *tot = reinterpret_cast<long long *>(wsb + a.off_tot) + ((int64_t)(row0 + j) * d + l) * 2;
                long long *totcnt = reinterpret_cast<long long *>(wsb + a.off_totcnt) + (int64_t)(row0 + j) * d + l;
                long long hi = tot[0];
                unsigned long long lo = (unsigned long long)tot[1];
                long long cnt = *totcnt;
                for (int sl = 0; sl < nsl; ++sl) {
                    const unsigned long long nlo = lo + part_lo[sl * E + e];
                    hi += part_hi[sl * E + e] + (nlo < lo ? 1 : 0);
                    lo = nlo;
                    cnt += part_cnt[sl * E + e];
                }
                tot[0] = hi;
                tot[1] = (long long)lo;
                *totcnt = cnt;
                int shift = colshift[l];
                if (colwide[l]) {
                    // total = main * 2^kLowBits + low, on the scale 2^-(shift + kLowBits)
                    const long long low = reinterpret_cast<const long long *>(wsb + a.off_losum)[(int64_t)(row0 + j) * d + l];
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
            cp = fmaf(c, scale, colmean[l]);     // (c - mean) * scale, one rounding, as for the points
        }
        cs[jj * DP + l] = cp;
        // operand position of (centroid j, feature l)
        const int qd = j >> 2, i = j & 3;
        const int t = qd / g.S, slot = rl * g.S + qd % g.S;
        const int m = 8 * (slot & 3) + 4 * (slot >> 2) + i;
        const int h = l / (DP / 2), sf = l % (DP / 2);
        unsigned short ph, pl;
        split2(-2.0f * cp, ph, pl);
        const int ks = sf >> 3, el = sf & 7, ln = h * 32 + m;
        opA[((int64_t)(t * NS + 0 * NK + ks) * 64 + ln) * 8 + el] = ph;
        opA[((int64_t)(t * NS + 1 * NK + ks) * 64 + ln) * 8 + el] = pl;
    }
    __syncthreads();
    float mx = 0.0f;
    if (tid < rows) {
        const int j = j0 + tid;
        float nrm = 0.0f;
        for (int l = 0; l < DP; ++l) nrm = fmaf(cs[tid * DP + l], cs[tid * DP + l], nrm);
        const int qd = j >> 2, i = j & 3;
        const int t = qd / g.S, slot = rl * g.S + qd % g.S;
        // bias slot, lower half-wave lane of this row: pieces of the squared norm
        unsigned ph, pm, pl;
        split3(nrm, ph, pm, pl);
        const int m = 8 * (slot & 3) + 4 * (slot >> 2) + i;
        unsigned short *bias = opA + ((int64_t)(t * NS + 2 * NK) * 64 + m) * 8;
        bias[0] = (unsigned short)ph; bias[1] = (unsigned short)pm; bias[2] = (unsigned short)pl;
        mx = nrm;
    }
    // rows <= 64: the first wave holds them all; the run's maximum is taken over its parts by the reader
    if (tid < 64) {
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        if (tid == 0) reinterpret_cast<float *>(wsb + a.off_cnmax)[run * kMaxParts + part] = mx;
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
    // eight loads in flight at a time (the walk is bound by their latency); the additions keep the chunk order
    constexpr int U = 8;
    for (int c0 = 0; c0 < n_chunks; c0 += U) {
        double t[U];
#pragma unroll
        for (int u = 0; u < U; ++u) t[u] = pj[(int64_t)min(c0 + u, n_chunks - 1) * n_runs + r];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (c0 + u < n_chunks) v = __dadd_rn(v, t[u]);
    }
    out[(int64_t)b * out_bs + (int64_t)r * out_stride + out_off] = v;
}

template <int DP>
hipError_t launch_sweep_dp(const SweepPlan &plan, const SweepLayout &L, const SweepArgs &a, hipStream_t s)
{
    // the kernels' LDS limit is raised once per process, whichever host thread comes first
    static std::once_flag attr_once;
    static hipError_t attr_status = hipSuccess;
    std::call_once(attr_once, [] {
        const void *fns[] = {
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, false, false, false>),
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, false, false, true>),
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, false, true, false>),
            reinterpret_cast<const void *>(lloyd_step_kernel<DP, true, false, false>),
        };
        for (const void *fn : fns) {
            const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) attr_status = e;
        }
    });
    if (attr_status != hipSuccess) return attr_status;
    const int batch = a.batch;
    // column statistics
    if (!a.reuse_colstats) {
        hipLaunchKernelGGL(colstats_kernel, dim3(L.stat_blocks, batch), dim3(kThreads), 0, s, a.X, a.N, (int)a.d, DP, a.ldx,
                           a.x_batch_stride, a.ws, L.per_batch, L.colstat_part);
        hipLaunchKernelGGL(colstats_final_kernel, dim3(batch), dim3(256), 0, s, a.N, (int)a.d, (int)L.stat_blocks, a.ws,
                           L.per_batch, L.colstat_part, L.colinfo, a.status);
    }
    // Rounds after the first run on the prepared copy of the points - unless the loss of every round is wanted (that
    // pass needs every row), or the sweep is so light in distance work (a single k up to 32: one tile of centroids per
    // group) that reading the rows is what it costs: the prepared copy is 6 to 12% larger than the rows.
    const bool trace = a.trace != nullptr;
    const bool use_pre = sweep_uses_prepared(plan, a.iters, trace);
    if (use_pre && !a.reuse_prepared) {
        // the prepared copy: one wave per block of 32 points, a few blocks per wave
        const int64_t n_blocks = (a.N + 31) / 32;
        int64_t grid_x = (n_blocks + 4 * 8 - 1) / (4 * 8);      // 4 waves per workgroup, ~8 blocks per wave
        if (grid_x > 4096) grid_x = 4096;
        if (grid_x < 1) grid_x = 1;
        hipLaunchKernelGGL((lloyd_prepare_kernel<DP>), dim3((unsigned)grid_x, batch), dim3(256), 0, s, a.X, a.N, (int)a.d, a.ldx,
                           a.x_batch_stride, a.status, a.ws, L.per_batch, L.colinfo, L.xp);
    }
    InitArgs ia;
    ia.ws = a.ws; ia.ws_bs = L.per_batch;
    ia.off_opA = L.opA; ia.off_losum = L.losum; ia.off_tot = L.tot; ia.off_totcnt = L.totcnt; ia.off_prev = L.prev;
    ia.n_tiles = plan.total_tiles; ia.dp = DP;
    ia.n_losum = (int64_t)plan.total_rows * a.d; ia.n_tot = ia.n_losum * 2; ia.n_totcnt = ia.n_losum;
    ia.n_prev16 = (int64_t)plan.lab_slots * align_up(a.N, 16) / 16;
    hipLaunchKernelGGL(sweep_init_kernel, dim3(512, batch), dim3(256), 0, s, ia);

    CentroidArgs ca;
    ca.X = a.X; ca.N = a.N; ca.d = a.d; ca.ldx = a.ldx; ca.x_bs = a.x_batch_stride;
    ca.init_idx = a.init_idx; ca.init_bs = a.init_batch_stride;
    ca.C = a.centroids; ca.c_bs = (int64_t)plan.total_rows * a.d;
    ca.status = a.status; ca.ws = a.ws; ca.ws_bs = L.per_batch;
    ca.off_colinfo = L.colinfo; ca.off_opA = L.opA; ca.off_cnmax = L.cnmax;
    ca.off_psum = L.psum; ca.off_pcnt = L.pcnt; ca.off_losum = L.losum; ca.off_tot = L.tot; ca.off_totcnt = L.totcnt;
    const dim3 centroid_grid(parts_upto(plan.k_min + plan.n_runs - 1) - parts_upto(plan.k_min - 1), batch);
    hipLaunchKernelGGL((lloyd_centroids_kernel<DP, true>), centroid_grid, dim3(kThreads), 0, s, plan, ca);

    StepArgs sa;
    sa.X = a.X; sa.N = a.N; sa.d = a.d; sa.ldx = a.ldx; sa.x_bs = a.x_batch_stride;
    sa.C = a.centroids; sa.c_bs = ca.c_bs;
    sa.labels = a.labels; sa.lab_bs = (int64_t)plan.n_runs * a.N;
    sa.status = a.status; sa.ws = a.ws; sa.ws_bs = L.per_batch;
    sa.off_colinfo = L.colinfo; sa.off_opA = L.opA; sa.off_cnmax = L.cnmax;
    sa.off_psum = L.psum; sa.off_pcnt = L.pcnt; sa.off_pj = L.pj; sa.off_losum = L.losum; sa.off_prev = L.prev;
    sa.off_xp = L.xp; sa.off_log = L.log;

    size_t lds = 0;
    for (int gi = 0; gi < plan.n_groups; ++gi) {
        const GroupDesc &g = plan.g[gi];
        const int rr = rows_before(plan.k_min, g.run0 + g.n_runs) - rows_before(plan.k_min, g.run0);
        const size_t need = (size_t)carve_lds(DP, a.d, g.n_tiles, rr, g.copies).total;
        if (need > lds) lds = need;
    }
    const dim3 grid((unsigned)((int64_t)plan.n_groups * plan.n_chunks * batch), 1);
    sa.batch = batch;
    const bool prof = profile_enabled();
    for (int t = 0; t < a.iters; ++t) {
        sa.first_round = t == 0 ? 1 : 0;
        if (prof) { hipError_t e = profile_mark(s, true); if (e != hipSuccess) return e; }
        if (trace) {
            hipLaunchKernelGGL((lloyd_step_kernel<DP, false, true, false>), grid, dim3(step_threads_of(DP)), lds, s, plan, sa);
            if (prof) { hipError_t e = profile_mark(s, false); if (e != hipSuccess) return e; }
            hipLaunchKernelGGL(lloyd_loss_kernel, dim3(batch), dim3(128), 0, s, plan.n_runs, plan.n_chunks, a.status, a.ws,
                               L.per_batch, L.pj, a.trace, (int64_t)plan.n_runs * (a.iters + 1), (int64_t)(a.iters + 1), (int64_t)t);
        } else {
            // the first round brings every row into a cluster and reads the rows themselves; later rounds take the
            // operands from the prepared copy and read a row only where a label is in doubt or has changed
            if (t == 0 || !use_pre) hipLaunchKernelGGL((lloyd_step_kernel<DP, false, false, false>), grid, dim3(step_threads_of(DP)), lds, s, plan, sa);
            else hipLaunchKernelGGL((lloyd_step_kernel<DP, false, false, true>), grid, dim3(step_threads_of(DP)), lds, s, plan, sa);
            if (prof) { hipError_t e = profile_mark(s, false); if (e != hipSuccess) return e; }
        }
        hipLaunchKernelGGL((lloyd_centroids_kernel<DP, false>), centroid_grid, dim3(kThreads), 0, s, plan, ca);
    }
    hipLaunchKernelGGL((lloyd_step_kernel<DP, true, false, false>), grid, dim3(step_threads_of(DP)), lds, s, plan, sa);
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

bool sweep_uses_prepared(const SweepPlan &plan, int32_t iters, bool trace)
{
    return !trace && iters >= 2 && plan.total_tiles >= 2 * plan.n_groups;
}

LloydGeometry lloyd_geometry(int dp)
{
    LloydGeometry g;
    g.threads = kThreads;
    g.tile_points = tile_points_of(dp);
    g.lds_budget = 156 * 1024;
    return g;
}

int64_t lloyd_group_lds_bytes(int dp, int d, int n_tiles, int real_rows, int copies)
{
    return carve_lds(dp, d, n_tiles, real_rows, copies).total;
}

constexpr int kFillWorkgroups = 256;   // one per compute unit

int32_t make_sweep_plan(int64_t N, int32_t d, int32_t k_min, int32_t k_max, int32_t batch, SweepPlan *plan)
{
    const int dp = padded_d(d);
    const LloydGeometry geo = lloyd_geometry(dp);
    plan->n_runs = k_max - k_min + 1;
    plan->k_min = k_min;
    plan->dp = dp;
    plan->n_groups = 0;
    int tiles = 0;
    int run = 0;
    int lab_slots = 0;       // run slots (8 / S per group) of the groups so far
    while (run < plan->n_runs) {
        // candidates: R runs side by side (8 / R slots each); take the one with the least padding per real
        // row, preferring the larger R - except between candidates that cover the same runs at the same padding
        // (the end of a range, a single k): there the smaller R wins, since a lane keeps state for R runs, used or not
        int best_R = 0, best_tiles = 0, best_nr = 0;
        double best_score = 1e30;
        for (int R = 8; R >= 1; R >>= 1) {
            const int S = 8 / R;
            const int nr = plan->n_runs - run < R ? plan->n_runs - run : R;
            const int kmax_g = k_min + run + nr - 1;
            const int quads = (kmax_g + 3) / 4;
            const int n_tiles = (quads + S - 1) / S;
            const int real_rows = rows_before(k_min, run + nr) - rows_before(k_min, run);
            if (n_tiles > 32) continue;
            if (lloyd_group_lds_bytes(dp, d, n_tiles, real_rows, 1) > geo.lds_budget) continue;
            // cost per real row: padded rows and a fixed per-group overhead
            const double score = (n_tiles * 32.0 + 24.0) / real_rows;
            if (score < best_score - 1e-12 || (nr == best_nr && score < best_score + 1e-12)) {
                best_score = score; best_R = R; best_tiles = n_tiles; best_nr = nr;
            }
        }
        if (best_R == 0 || plan->n_groups >= kMaxGroups) return RLS_ERR_INVALID_ARG;
        GroupDesc &g = plan->g[plan->n_groups++];
        g.run0 = (int16_t)run; g.n_runs = (int16_t)best_nr; g.S = (int16_t)(8 / best_R); g.n_tiles = (int16_t)best_tiles;
        g.lab0 = (int16_t)lab_slots; g.tile0 = tiles;
        lab_slots += best_R;
        // Runs with few clusters send many lanes of a wave to the same accumulator address (32 / k on average), which
        // the LDS works off one after the other: such groups keep several copies of their accumulators, LDS permitting.
        {
            const int kmax_g = k_min + run + best_nr - 1;
            const int real_rows = rows_before(k_min, run + best_nr) - rows_before(k_min, run);
            int copies = kmax_g <= 8 ? 16 : (kmax_g <= 16 ? 8 : (kmax_g <= 32 ? 4 : (kmax_g <= 64 ? 2 : 1)));
            while (copies > 1 && lloyd_group_lds_bytes(dp, d, best_tiles, real_rows, copies) > geo.lds_budget) copies >>= 1;
            g.copies = (int16_t)copies;
        }
        tiles += best_tiles;
        run += best_nr;
    }
    plan->total_tiles = tiles;
    plan->lab_slots = lab_slots;
    // launch order: groups by falling cost (tiles per point)
    for (int i = 0; i < plan->n_groups; ++i) plan->sched[i] = (uint8_t)i;
    for (int i = 1; i < plan->n_groups; ++i) {
        const uint8_t v = plan->sched[i];
        int j = i;
        while (j > 0 && plan->g[plan->sched[j - 1]].n_tiles < plan->g[v].n_tiles) { plan->sched[j] = plan->sched[j - 1]; --j; }
        plan->sched[j] = v;
    }
    plan->total_rows = rows_before(k_min, plan->n_runs);
    // chunks: enough workgroups over the whole batch to fill the chip twice over (a workgroup stages its
    // group's rows once, so more and shorter chunks only add set-up); a chunk never exceeds 2^16 points (the accumulators
    // would allow 2^17; with the groups of a chunk running side by side the shorter chunk measured 2% shorter launches at 8M x 32)
    const int tp = geo.tile_points;
    const int64_t tiles_total = (N + tp - 1) / tp;
    const int64_t units = (int64_t)plan->n_groups * (batch > 0 ? batch : 1);
    int64_t want = (512 + units - 1) / units;       // two workgroups per compute unit (1024 measured 4% longer launches at 1M x 16, 256 22% longer)
    // a workgroup should have several slabs per wave to spread its set-up over: at least 4096 points per chunk
    // but never fewer workgroups than fill the chip
    int64_t most = (N + 4095) / 4096;
    const int64_t fill = (kFillWorkgroups + units - 1) / units;
    if (most < fill) most = fill;
    if (want > most) want = most;
    if (want > tiles_total) want = tiles_total;
    if (want < 1) want = 1;
    int64_t chunk_len = ((tiles_total + want - 1) / want) * tp;
    const int64_t cap = (int64_t)1 << 16;
    if (chunk_len > cap) chunk_len = cap / tp * tp;
    plan->chunk_len = (int32_t)chunk_len;
    plan->n_chunks = (int32_t)((N + chunk_len - 1) / chunk_len);
    // chunks per block of the launch order: about one workgroup per compute unit in a block, a multiple of eight chunks
    // (workgroups go to the eight XCDs in turn, so the groups of one chunk meet on one XCD)
    int32_t cb = (kFillWorkgroups + plan->n_groups - 1) / plan->n_groups;
    cb = (cb + 7) / 8 * 8;
    const int64_t n_all = (int64_t)plan->n_chunks * (batch > 0 ? batch : 1);     // chunks of all spaces of the batch
    if (cb > n_all) cb = (int32_t)n_all;
    plan->chunk_block = cb;
    if ((int64_t)plan->n_groups * n_all > 0x7fffffffLL) return RLS_ERR_INVALID_ARG;
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
    L->near = take(N);
    L->seedthr = take((int64_t)k_max * 8);
    L->xp = take((N + 31) / 32 * prep_block_u4_of(plan.dp) * 16);     // (with the blocks above: the same place whatever the range of k)
    L->opA = take((int64_t)plan.total_tiles * tile_bytes_of(plan.dp));
    L->cnmax = take((int64_t)plan.n_runs * kMaxParts * 4);
    L->psum = take((int64_t)plan.n_chunks * plan.total_rows * d * 8);
    L->pcnt = take((int64_t)plan.n_chunks * plan.total_rows * 4);
    L->pj = take((int64_t)plan.n_chunks * plan.n_runs * 8);
    L->losum = take((int64_t)plan.total_rows * d * 8);
    L->tot = take((int64_t)plan.total_rows * d * 16);
    L->totcnt = take((int64_t)plan.total_rows * d * 8);
    L->prev = take((int64_t)plan.lab_slots * align_up(N, 16));
    L->log = take((int64_t)plan.n_groups * plan.n_chunks * (step_threads_of(plan.dp) / 64) * kLogCap * 8);
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
