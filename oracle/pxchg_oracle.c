/*
 * CPU oracle for the per-GPU arithmetic of the parameter exchange.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the exchange computes, as
 * scalar loops, one element at a time, in the order the paper's exchange is
 * stated.  It is slow on purpose and is never part of the product path: only
 * the tests, the smoke check and the CPU-baseline leg of the benchmark may call
 * it.  It shares no code, header, table or constant with the HIP library.
 *
 * What the paper fixes (Section 3.2): every rank receives all k ranks' copies
 * of its slice, sums them on the GPU ("Alltoall-sum-Allgather"), and the
 * half-precision variant moves the data as 16-bit floats while the sum itself
 * is carried out at full (32-bit) precision.  Section 4 fixes what is summed:
 * parameter updates/gradients before descent (SUBGD), or weights and momentum
 * after it (AWAGD, an average), with momentum SGD as the optimiser, and the
 * elastic-averaging update with moving rate alpha for the asynchronous mode.
 * The paper prints none of the formulas; the readings taken are stated at each
 * function.
 *
 * Precision: the method's own precision is binary32 with a binary16 wire
 * format, so the oracle computes in `float` with every operation rounded
 * separately.  Build with -ffp-contract=off and without fast-math.
 *
 * Parity pins (tests/test_oracle_*.py): binary16 conversion against the
 * IEEE-754 definition (exhaustive widen/narrow round trip, every tie between
 * adjacent halves, range boundaries) and against numpy's own conversion; the
 * sum against exact rational arithmetic and order-sensitive hand cases; the
 * momentum update against its closed form and torch.optim.SGD on the CPU; the
 * elastic update against conservation, midpoint and geometric-decay closed
 * forms; the tree-ordered sum of squares against hand-derived cases in which
 * the owner of an element (lane, wavefront, block) decides a rounding, against
 * the index-order sum where every order is exact, and against the exactly
 * rounded sum within the bound of a binary64 sum.  No function here is unpinned.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_F16 = 1 };
enum { ORACLE_AVG = 0, ORACLE_SUM = 1 };

static uint32_t bits_of(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float float_of(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/*
 * binary32 -> binary16, round to nearest, ties to even (the reduced-precision
 * transfer of Section 3.2; the paper says only "half precision", IEEE's default
 * rounding is the reading).  Works on the bit patterns:
 *   - NaN stays NaN (sign kept, quiet bit set, top payload bits kept);
 *   - magnitudes that round to 2^16 or more become infinity;
 *   - results below 2^-14 are binary16 subnormals (gradual underflow);
 *   - magnitudes of 2^-25 or less round to zero, sign kept.
 */
uint16_t oracle_f32_to_f16_bits(uint32_t x)
{
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t mag = x & 0x7fffffffu;

    if (mag >= 0x7f800000u) {                 /* infinity or NaN */
        if (mag == 0x7f800000u) return (uint16_t)(sign | 0x7c00u);
        return (uint16_t)(sign | 0x7e00u | ((mag >> 13) & 0x01ffu));
    }
    int32_t e = (int32_t)(mag >> 23) - 127;   /* unbiased exponent */
    uint32_t m = mag & 0x007fffffu;

    if (e >= 16) return (uint16_t)(sign | 0x7c00u);

    if (e >= -14) {                           /* lands in the normal range */
        uint32_t h = ((uint32_t)(e + 15) << 10) | (m >> 13);
        uint32_t rest = m & 0x1fffu;          /* the 13 bits dropped */
        if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1u;
        /* a carry out of the mantissa bumps the exponent; 0x7c00 is infinity */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign;                 /* below half the smallest subnormal */

    /* subnormal result: value = M * 2^(e-23) with M the 24-bit significand,
     * to be expressed in units of 2^-24, so shift right by (-e - 1) bits. */
    uint32_t M = m | 0x00800000u;
    int shift = -e - 1;                       /* 14 .. 24 */
    uint32_t h = M >> shift;
    uint32_t rest = M & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rest > half || (rest == half && (h & 1u))) h += 1u;
    return (uint16_t)(sign | h);              /* h == 0x0400 is the smallest normal */
}

/* binary16 -> binary32: exact for every input (Section 3.2: the sum is done at
 * full precision, so received halves are widened first). */
uint32_t oracle_f16_to_f32_bits(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t e = ((uint32_t)h >> 10) & 0x1fu;
    uint32_t m = (uint32_t)h & 0x03ffu;

    if (e == 0x1fu) return sign | 0x7f800000u | (m << 13);       /* inf / NaN */
    if (e != 0) return sign | ((e + 112u) << 23) | (m << 13);     /* normal */
    if (m == 0) return sign;                                      /* zero */
    /* subnormal: m * 2^-24; normalise */
    int p = 9;
    while (!(m & (1u << p))) --p;            /* top set bit of m, 0..9 */
    uint32_t frac = (m << (23 - p)) & 0x007fffffu;
    return sign | ((uint32_t)(p - 24 + 127) << 23) | frac;
}

static float widen(uint16_t h) { return float_of(oracle_f16_to_f32_bits(h)); }
static uint16_t narrow(float f) { return oracle_f32_to_f16_bits(bits_of(f)); }

/* Step "pack": h[j] = half(g[j]) (Section 3.2, half-precision transfer). */
void oracle_pack_fp16(const float *g, uint16_t *h, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) h[j] = narrow(g[j]);
}

/* Step "unpack": exact widening of what was received. */
void oracle_unpack_fp16(const uint16_t *h, float *g, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) g[j] = widen(h[j]);
}

/*
 * Step "sum" of Alltoall-sum-Allgather (Section 3.2), on one rank's slice:
 *   s = c_0[j];  s = s + c_i[j] for i = 1 .. k-1, in worker order, in binary32,
 *   rounded after every addition (halves are widened exactly first);
 *   mode AVG: a = s / (float)k, one correctly rounded division (the average of
 *   Section 4's weight averaging, and the 1/k of averaged gradients);
 *   mode SUM: a = s (Section 4's summed updates, taken literally);
 *   the result leaves as binary32, or rounded once to binary16 for the second
 *   transfer leg.
 * The running sum starts from c_0 itself, not from zero, so a lone -0 stays -0.
 */
int oracle_reduce_avg(int k, const void *const *contrib, int in_dtype,
                      void *out, int out_dtype, int mode, int64_t n)
{
    if (k < 1 || !contrib || !out || n < 0) return 1;
    if ((in_dtype != ORACLE_F32 && in_dtype != ORACLE_F16) ||
        (out_dtype != ORACLE_F32 && out_dtype != ORACLE_F16) ||
        (mode != ORACLE_AVG && mode != ORACLE_SUM)) return 1;
    const float kf = (float)k;
    for (int64_t j = 0; j < n; ++j) {
        float s;
        if (in_dtype == ORACLE_F32) {
            s = ((const float *)contrib[0])[j];
            for (int i = 1; i < k; ++i) s = s + ((const float *)contrib[i])[j];
        } else {
            s = widen(((const uint16_t *)contrib[0])[j]);
            for (int i = 1; i < k; ++i) s = s + widen(((const uint16_t *)contrib[i])[j]);
        }
        float a = (mode == ORACLE_AVG) ? s / kf : s;
        if (out_dtype == ORACLE_F32) ((float *)out)[j] = a;
        else ((uint16_t *)out)[j] = narrow(a);
    }
    return 0;
}

/*
 * Momentum SGD (Section 4 names the optimiser, prints no formula).  Reading:
 * the form of the AlexNet paper the report builds on, weight decay folded into
 * the gradient:
 *      gg = a + wd * w
 *      v' = mu * v - lr * gg
 *      w' = w + v'
 * `a` is the exchanged gradient, binary32 or binary16 (widened exactly).
 * Every product, sum and difference is rounded to binary32 on its own.
 */
int oracle_sgd_momentum(const void *a, int a_dtype, float *w, float *v,
                        float lr, float mu, float wd, int64_t n)
{
    if (!a || !w || !v || n < 0) return 1;
    if (a_dtype != ORACLE_F32 && a_dtype != ORACLE_F16) return 1;
    for (int64_t j = 0; j < n; ++j) {
        float g = (a_dtype == ORACLE_F32) ? ((const float *)a)[j]
                                          : widen(((const uint16_t *)a)[j]);
        float dw = wd * w[j];
        float gg = g + dw;
        float mv = mu * v[j];
        float lg = lr * gg;
        float vn = mv - lg;
        v[j] = vn;
        w[j] = w[j] + vn;
    }
    return 0;
}

/*
 * Elastic averaging between one worker's parameters x and the center c
 * (Section 4, asynchronous mode, moving rate alpha; formula not printed).
 * Reading: the symmetric elastic pull with the same alpha on both sides,
 *      d = alpha * (x - c);   x' = x - d;   c' = c + d
 * each operation rounded to binary32.  Workers meet the center one at a time,
 * so a round is k calls in arrival order with c carried from one to the next.
 */
int oracle_easgd(float *x, float *c, float alpha, int64_t n)
{
    if (!x || !c || n < 0) return 1;
    for (int64_t j = 0; j < n; ++j) {
        float diff = x[j] - c[j];
        float d = alpha * diff;
        x[j] = x[j] - d;
        c[j] = c[j] + d;
    }
    return 0;
}

/*
 * Diagnostics of one exchanged buffer, for watching the reduced-precision
 * transfer (Section 4 reports an accuracy cost of the half-precision exchange):
 * how many elements are not finite (an overflow in the pack shows up as an
 * infinity), the largest finite magnitude, and the sum of squares of the finite
 * elements accumulated in binary64 in index order (its square root is the
 * L2 norm).  Elements are binary32, or binary16 widened exactly.
 */
int oracle_stats(const void *a, int dtype, int64_t n, uint64_t *nonfinite, float *max_abs, double *sum_sq)
{
    if (!a || n < 0 || !nonfinite || !max_abs || !sum_sq) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_F16) return 1;
    uint64_t bad = 0;
    float mx = 0.0f;
    double ss = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        float x = (dtype == ORACLE_F32) ? ((const float *)a)[j] : widen(((const uint16_t *)a)[j]);
        if ((bits_of(x) & 0x7f800000u) == 0x7f800000u) {   /* infinity or NaN */
            ++bad;
            continue;
        }
        float ax = x < 0.0f ? -x : x;
        if (ax > mx) mx = ax;
        ss = ss + (double)x * (double)x;
    }
    *nonfinite = bad;
    *max_abs = mx;
    *sum_sq = ss;
    return 0;
}

/*
 * The same diagnostics with the sum of squares taken in a FIXED TREE ORDER, so
 * that a parallel implementation can reproduce it bit for bit run after run
 * (a binary64 sum in index order cannot be parallelised without changing its
 * rounding).  The paper defines no such quantity (Section 4 only reports what
 * the half-precision exchange costs in accuracy); the order below is this
 * library's definition, stated in its header, and written out here with plain
 * loops.  `waves`, `block_chunks` and `combine_threads` are parameters of that
 * definition, not of an implementation.
 *
 *   Work list.  Tensor t is cut into chunks of at most chunk_elems consecutive
 *   elements, tensors in order, empty tensors giving none; chunks are numbered
 *   g = 0, 1, ... over the whole list.  `block_chunks` consecutive chunks form
 *   block b = g / block_chunks; j = g % block_chunks is the chunk's place in it.
 *
 *   Accumulators.  A block has waves x 64 of them, all starting at +0.
 *   Element i of a chunk (i counted from the chunk's start) belongs to
 *   accumulator (wave, lane) = (j % waves, (i / piece) % 64), where `piece` is
 *   the number of elements in 16 bytes (4 for binary32, 8 for binary16).  An
 *   accumulator takes its elements in increasing (g, i): acc = acc + x*x, the
 *   square exact in binary64, the sum rounded once.  Elements that are not
 *   finite are counted and add nothing.
 *
 *   combine(values[0..n), T), T a multiple of 64: "thread" t adds values t,
 *   t + T, t + 2T, ... in that order onto +0; the 64 threads of each group
 *   t / 64 then exchange in a butterfly, a[l] = a[l] + a[l ^ off] for off = 32,
 *   16, 8, 4, 2, 1 (all 64 at once per step), after which a[0] is the group's
 *   value; the groups' values are added in group order, starting from group 0's.
 *
 *   A block's sum is combine(its accumulators in (wave, lane) order, waves*64);
 *   the result is combine(the blocks' sums in block order, combine_threads).
 *
 * The count and the maximum are exact in any order.
 */
static double ordered_combine(const double *values, int64_t n, int threads)
{
    double *a = (double *)calloc((size_t)threads, sizeof(double));
    double tmp[64];
    double total = 0.0;
    if (!a) return -1.0;
    for (int t = 0; t < threads; ++t)
        for (int64_t i = t; i < n; i += threads) a[t] = a[t] + values[i];
    for (int grp = 0; grp < threads / 64; ++grp) {
        double *lane = a + 64 * grp;
        for (int off = 32; off >= 1; off /= 2) {
            for (int l = 0; l < 64; ++l) tmp[l] = lane[l] + lane[l ^ off];
            memcpy(lane, tmp, sizeof(tmp));
        }
        total = (grp == 0) ? lane[0] : total + lane[0];
    }
    free(a);
    return total;
}

int oracle_stats_ordered(int n_tensors, const void *const *tensors, const int64_t *counts, int dtype,
                         int64_t chunk_elems, int waves, int block_chunks, int combine_threads,
                         uint64_t *nonfinite, float *max_abs, double *sum_sq)
{
    if (n_tensors < 1 || !tensors || !counts || !nonfinite || !max_abs || !sum_sq) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_F16) return 1;
    if (chunk_elems < 1 || waves < 1 || block_chunks < 1 || combine_threads < 64 || combine_threads % 64) return 1;
    const int piece = (dtype == ORACLE_F32) ? 4 : 8;
    int64_t n_chunks = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (counts[t] < 0 || (counts[t] > 0 && !tensors[t])) return 1;
        n_chunks += (counts[t] + chunk_elems - 1) / chunk_elems;
    }
    const int64_t n_blocks = (n_chunks + block_chunks - 1) / block_chunks;
    double *block_sum = (double *)calloc((size_t)(n_blocks > 0 ? n_blocks : 1), sizeof(double));
    double *acc = (double *)calloc((size_t)waves * 64, sizeof(double));
    if (!block_sum || !acc) { free(block_sum); free(acc); return 1; }

    uint64_t bad = 0;
    float mx = 0.0f;
    int64_t g = 0;                               /* running chunk number */
    for (int t = 0; t < n_tensors; ++t) {
        for (int64_t start = 0; start < counts[t]; start += chunk_elems, ++g) {
            const int64_t len = counts[t] - start < chunk_elems ? counts[t] - start : chunk_elems;
            const int j = (int)(g % block_chunks);
            double *wave_acc = acc + 64 * (j % waves);
            for (int64_t i = 0; i < len; ++i) {
                float x = (dtype == ORACLE_F32) ? ((const float *)tensors[t])[start + i]
                                                : widen(((const uint16_t *)tensors[t])[start + i]);
                const int finite = (bits_of(x) & 0x7f800000u) != 0x7f800000u;   /* neither infinity nor NaN */
                if (!finite) { ++bad; continue; }
                float mag = x < 0.0f ? -x : x;
                if (mag > mx) mx = mag;
                double *slot = wave_acc + (i / piece) % 64;
                *slot = *slot + (double)x * (double)x;
            }
            if (j == block_chunks - 1 || g == n_chunks - 1) {    /* the block is complete */
                block_sum[g / block_chunks] = ordered_combine(acc, (int64_t)waves * 64, waves * 64);
                memset(acc, 0, (size_t)waves * 64 * sizeof(double));
            }
        }
    }
    *nonfinite = bad;
    *max_abs = mx;
    *sum_sq = ordered_combine(block_sum, n_blocks, combine_threads);
    free(block_sum);
    free(acc);
    return 0;
}
