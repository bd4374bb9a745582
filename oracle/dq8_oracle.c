/*
 * dq8 CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct implementation of the 8-bit approximation
 * codec of "8-Bit Approximations for Parallelism in Deep Learning"
 * (arXiv 1511.04561): codebooks (Sec. 3.1), absmax normalisation (Sec. 3.1,
 * last paragraph), nearest-code compression and table-lookup decompression
 * (Sec. 3.2), and the averaging of worker buffers that data parallelism
 * performs on the decompressed values (Sec. 2.1).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, table or constant with the HIP library and
 * includes none of its headers.  Nothing here is tuned: the encoder is a
 * brute-force scan over all 256 codes per element.
 *
 * Arithmetic contract (build with -O2 -fno-fast-math -ffp-contract=off,
 * default rounding mode, no flush-to-zero):
 *   - every fp32 operation (divide, multiply, add) is a single IEEE-754
 *     binary32 round-to-nearest-even operation; no fused multiply-add;
 *   - codebook entries are exact small integer ratios evaluated with one
 *     fp64 division and then rounded to fp32;
 *   - distances in the nearest-code search are fp64 (exact for every pair of
 *     candidates that can compete, see nearest_code).
 *
 * Parity status: every function below is pinned by tests that do not reuse
 * its formula (bit-by-bit tree walk in exact rationals, sorted-table search,
 * exact rational rounding, numpy primitives, brute force on tiny inputs,
 * error bounds, and the relative-error ordering of the paper's Table 2).
 * The average with a local 32-bit term and the average-then-compress round
 * are pinned the same way (numpy and exact-rational re-computation, special
 * cases with closed-form results); where the local term sits in the sum and
 * that the divisor is K + 1 is a reading of one sentence of Sec. 3.4.
 * The error statistics (Sec. 3.4, Table 2) are pinned by exact rational sums,
 * the quarter-step closed form of uniform quantisation, special cases,
 * additivity over blocks and a band around the 16 relative errors the paper
 * prints for synthetic samples; that zeros are left out of the relative mean is
 * a reading (the paper does not say).
 * What is NOT pinned, because the paper prints no table values and its
 * figure of the bit layouts is missing: agreement with the bit patterns of
 * the authors' own implementation ("parity unpinned" for wire compatibility
 * with that code; none is claimed).
 */
#include <float.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#if !defined(FLT_EVAL_METHOD) || FLT_EVAL_METHOD != 0
#error "float expressions must be evaluated in binary32 (FLT_EVAL_METHOD == 0)"
#endif
#if defined(__FAST_MATH__) || defined(__FP_FAST_FMAF)
#error "build the oracle without fast-math and without FMA contraction"
#endif

enum { DQ8O_DYNAMIC_TREE = 0, DQ8O_LINEAR = 1, DQ8O_STATIC_TREE = 2, DQ8O_MANTISSA = 3 };

static int g_threads = 1; /* used only to time the oracle; results do not depend on it */

int dq8o_set_threads(int t)
{
    if (t < 1) t = 1;
#ifdef _OPENMP
    g_threads = t;
#else
    g_threads = 1;
#endif
    return g_threads;
}

int dq8o_get_threads(void) { return g_threads; }

/*
 * Sec. 3.1: one sign bit, seven bits of magnitude.  Magnitude index j = code & 127
 * is ascending in value, code bit 7 is the sign, so cb[j + 128] = -cb[j].
 *
 * Dynamic tree (Sec. 3.1, third paragraph): the 7-bit field holds n leading zero
 * bits (decimal exponent 10^-n), a flag bit set to one, and t = 6 - n tree bits.
 * The tree bisects the interval (0.1, 1): t bits select one of 2^t equal pieces,
 * piece k spans 0.1 + 0.9 k / 2^t .. 0.1 + 0.9 (k+1) / 2^t, and the value is the
 * middle of that piece times 10^-n:
 *     (0.1 + 0.9 (k + 1/2) / 2^t) 10^-n = (2^(t+1) + 9 (2k+1)) / (2^(t+1) 10^(n+1)).
 * The all-zero field has no flag and stands for exactly zero.
 *
 * Linear quantisation (Sec. 3.1, last paragraph; Sec. 4.1): 128 equally spaced
 * magnitudes on [0, 1] including both ends: j / 127.
 *
 * Static tree (Sec. 3.1, second paragraph): 3-bit exponent field E and a 4-bit
 * bisection tree over (0.1, 1).  The exponent is stored so that a larger field is
 * a larger value: decade 10^(E-7), value (0.1 + 0.9 (k + 1/2) / 16) 10^(E-7)
 *     = (32 + 9 (2k+1)) / (32 10^(8-E)).
 * This type has no zero.
 *
 * Mantissa type (Sec. 3.1, first paragraph: with a 3-bit exponent the mantissa
 * holds the values 0 to 15): 3-bit exponent field E, 4-bit mantissa m, value
 * m 10^(E-8) = m / 10^(8-E), the same decades as the static tree (whose tree
 * covers 0.1 .. 1 of 10^(E-7)).  Several fields stand for the same value: m = 0
 * is zero for every E, and m = 10 of one decade equals m = 1 of the next.
 */
int dq8o_codebook(int kind, float *cb)
{
    int j;
    if (!cb) return 1;
    for (j = 0; j < 128; ++j) {
        double num, den;
        if (kind == DQ8O_DYNAMIC_TREE) {
            if (j == 0) {
                num = 0.0;
                den = 1.0;
            } else {
                int len = 0, n, t, k, e;
                while ((j >> len) != 0) ++len; /* position of the flag bit + 1 */
                n = 7 - len;                   /* leading zeros in the 7-bit field */
                t = 6 - n;                     /* tree bits after the flag */
                k = j - (1 << t);              /* tree path read as an integer */
                num = (double)((1 << (t + 1)) + 9 * (2 * k + 1));
                den = (double)(1 << (t + 1));
                for (e = 0; e < n + 1; ++e) den *= 10.0; /* exact: at most 128e7 */
            }
        } else if (kind == DQ8O_LINEAR) {
            num = (double)j;
            den = 127.0;
        } else if (kind == DQ8O_STATIC_TREE) {
            int E = j >> 4, k = j & 15, e;
            num = (double)(32 + 9 * (2 * k + 1));
            den = 32.0;
            for (e = 0; e < 8 - E; ++e) den *= 10.0; /* exact: at most 32e8 */
        } else if (kind == DQ8O_MANTISSA) {
            int E = j >> 4, m = j & 15, e;
            num = (double)m;
            den = 1.0;
            for (e = 0; e < 8 - E; ++e) den *= 10.0; /* exact: at most 1e8 */
        } else {
            return 2;
        }
        cb[j] = (float)(num / den);
        cb[j + 128] = -cb[j];
    }
    return 0;
}

static size_t block_len(size_t n, size_t block) { return block == 0 ? n : block; }

/* Sec. 3.1, last paragraph: the scale of a block is its absolute maximum. */
static float block_absmax(const float *x, size_t lo, size_t hi)
{
    float s = 0.0f;
    size_t i;
    for (i = lo; i < hi; ++i) {
        float a = fabsf(x[i]);
        if (a > s) s = a;
    }
    return s;
}

int dq8o_absmax(const float *x, size_t n, size_t block, float *scales)
{
    size_t B, nb;
    long long b;
    if (n == 0) return 0;
    if (!x || !scales) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n;
        scales[b] = block_absmax(x, lo, hi);
    }
    return 0;
}

/*
 * Nearest code to the normalised value xn, scanning all 256 codes.
 * Distance is |xn - cb[c]| in fp64.  Two different magnitudes can only compete
 * when they are neighbours in the table; neighbouring table values and any xn
 * between them are binary32 numbers within a factor of a few of each other, so
 * their difference is exact in fp64 and the comparison of distances is the
 * comparison of the real distances.
 * Tie rules: equal distance -> the code of smaller magnitude; equal magnitude as
 * well (+v / -v when xn is a zero or rounds to a tie, or the two zeros) -> the
 * code whose sign bit equals the sign bit of xn; and among codes of one sign that
 * stand for the same value (the mantissa type has such) -> the smallest code.
 */
static uint8_t nearest_code(const float *cb, float xn)
{
    int c, best = -1;
    double bd = 0.0, bm = 0.0;
    int sx = signbit(xn) ? 1 : 0;
    for (c = 0; c < 256; ++c) {
        double d = fabs((double)xn - (double)cb[c]);
        double m = fabs((double)cb[c]);
        int better;
        if (best < 0)
            better = 1;
        else if (d != bd)
            better = d < bd;
        else if (m != bm)
            better = m < bm;
        else
            better = ((c >> 7) == sx) && ((best >> 7) != sx);
        if (better) {
            best = c;
            bd = d;
            bm = m;
        }
    }
    return (uint8_t)best;
}

/*
 * Compression (Sec. 3.1 last paragraph + Sec. 3.2): divide by the block's absolute
 * maximum, then take the nearest table value, keeping the sign.  A block whose
 * maximum is zero holds only zeros and is not divided.
 * scales_given != 0: scales[] is an input (one value per block) instead of being
 * computed here.
 */
int dq8o_encode(int kind, const float *x, size_t n, size_t block, float *scales,
                uint8_t *codes, int scales_given)
{
    float cb[256];
    size_t B, nb;
    long long b;
    int rc = dq8o_codebook(kind, cb);
    if (rc) return rc;
    if (n == 0) return 0;
    if (!x || !scales || !codes) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n, i;
        float s = scales_given ? scales[b] : block_absmax(x, lo, hi);
        if (!scales_given) scales[b] = s;
        for (i = lo; i < hi; ++i) {
            float xn; /* one binary32 rounding of the quotient */
            if (s == 0.0f)
                xn = x[i];
            else
                xn = x[i] / s;
            codes[i] = nearest_code(cb, xn);
        }
    }
    return 0;
}

/* Decompression (Sec. 3.2, third paragraph; Sec. 3.1, last paragraph):
 * look the code up in the table and multiply by the block's absolute maximum. */
int dq8o_decode(int kind, const uint8_t *codes, const float *scales, size_t n,
                size_t block, float *out)
{
    float cb[256];
    size_t B, nb;
    long long b;
    int rc = dq8o_codebook(kind, cb);
    if (rc) return rc;
    if (n == 0) return 0;
    if (!codes || !scales || !out) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n, i;
        float s = scales[b];
        for (i = lo; i < hi; ++i) {
            out[i] = cb[codes[i]] * s;
        }
    }
    return 0;
}

/*
 * Averaging of K workers' buffers (Sec. 2.1: parameters are synchronised by
 * averaging the exchanged gradients): decompress each worker's value, add them in
 * worker order 0..K-1 starting from +0, divide by K.  Each multiply, add and the
 * final divide is rounded to binary32 on its own.
 */
int dq8o_decode_accumulate_avg(int kind, const uint8_t *const *codes,
                               const float *const *scales, int K, size_t n,
                               size_t block, float *out)
{
    float cb[256];
    size_t B, nb;
    long long b;
    int k, rc = dq8o_codebook(kind, cb);
    if (rc) return rc;
    if (K < 1) return 3;
    if (n == 0) return 0;
    if (!codes || !scales || !out) return 1;
    for (k = 0; k < K; ++k)
        if (!codes[k] || !scales[k]) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n, i;
        for (i = lo; i < hi; ++i) {
            float acc = 0.0f;
            int kk;
            for (kk = 0; kk < K; ++kk) {
                float v = cb[codes[kk][i]] * scales[kk][b];
                acc = acc + v;
            }
            out[i] = acc / (float)K;
        }
    }
    return 0;
}

/*
 * Averaging with the worker's own 32-bit gradient (Sec. 3.4, MNIST paragraph: the
 * incoming buffers of the other GPUs are 8-bit approximations, the local GPU's own
 * gradient stays in 32 bits).  Reading taken here: the local value is the first
 * term of the same running sum, the K decompressed buffers follow in worker order,
 * and the divisor is the number of terms, K + 1:
 *     acc = +0;  acc = acc + local[i];  acc = acc + cb[code_k] * scale_k (k = 0..K-1);
 *     out = acc / (K + 1)
 * with every operation rounded to binary32 on its own.  K = 0 is allowed (the
 * local gradient alone).
 */
int dq8o_decode_accumulate_avg_local(int kind, const uint8_t *const *codes,
                                     const float *const *scales, int K, const float *local,
                                     size_t n, size_t block, float *out)
{
    float cb[256];
    size_t B, nb;
    long long b;
    int k, rc = dq8o_codebook(kind, cb);
    if (rc) return rc;
    if (K < 0) return 3;
    if (n == 0) return 0;
    if (!local || !out || (K > 0 && (!codes || !scales))) return 1;
    for (k = 0; k < K; ++k)
        if (!codes[k] || !scales[k]) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n, i;
        for (i = lo; i < hi; ++i) {
            float acc = 0.0f;
            int kk;
            acc = acc + local[i];
            for (kk = 0; kk < K; ++kk) {
                float v = cb[codes[kk][i]] * scales[kk][b];
                acc = acc + v;
            }
            out[i] = acc / (float)(K + 1);
        }
    }
    return 0;
}

/*
 * Second round of the gradient exchange (Appendix, cluster model: the gradients
 * are distributed once raw and once accumulated): the owner of a slice averages
 * the K received buffers (with its own 32-bit gradient when local != NULL) and
 * compresses the average again for redistribution.  By definition this is the
 * averaging above followed by the compression above, applied to the binary32
 * averages; nothing is fused or reordered here.
 */
int dq8o_decode_avg_encode(int kind, const uint8_t *const *codes, const float *const *scales,
                           int K, const float *local, size_t n, size_t block,
                           float *out_scales, uint8_t *out_codes)
{
    float cb[256];
    float *mean;
    int rc = dq8o_codebook(kind, cb); /* only to reject an unknown kind when n == 0 */
    if (rc) return rc;
    if (n == 0) return 0;
    if (!out_scales || !out_codes) return 1;
    mean = (float *)malloc(n * sizeof(float));
    if (!mean) return 4;
    if (local)
        rc = dq8o_decode_accumulate_avg_local(kind, codes, scales, K, local, n, block, mean);
    else
        rc = dq8o_decode_accumulate_avg(kind, codes, scales, K, n, block, mean);
    if (!rc) rc = dq8o_encode(kind, mean, n, block, out_scales, out_codes, 0);
    free(mean);
    return rc;
}


/*
 * Approximation error of a data type on a sample (Sec. 3.4, first paragraph and
 * Table 2: mean absolute and mean relative error of compress-then-decompress;
 * the tree and linear types normalise by the absolute maximum, the static types
 * may instead be given a fixed decade as the scale).  For every block b:
 *     q_i      = cb[code_i] * s_b              (binary32, as dq8o_decode)
 *     e_i      = | (double) q_i - (double) x_i |
 *     stats[4b+0] = sum of e_i over the block
 *     stats[4b+1] = sum of e_i / |x_i| (each quotient one binary64 division) over
 *                   the elements with x_i != 0
 *     stats[4b+2] = number of elements with x_i != 0
 *     stats[4b+3] = largest e_i
 * The paper does not say what the relative error of a zero is; here zeros are
 * left out of that sum and counted, so that the caller divides by the number of
 * terms.  Sums run over the block in index order in long double (64-bit
 * significand on this target), so they are far closer to the real sums than any
 * binary64 summation; only the last step rounds to binary64.
 * means (may be NULL): means[0] = (sum of all e_i) / n, means[1] = (sum of all
 * relative errors) / (number of non-zero x_i), or 0 when there is none; block
 * sums are added in block order in long double.
 */
int dq8o_error_stats(int kind, const float *x, size_t n, size_t block, float *scales,
                     int scales_given, double *stats, double *means)
{
    float cb[256];
    size_t B, nb;
    long long b;
    long double *part;
    int rc = dq8o_codebook(kind, cb);
    if (rc) return rc;
    if (n == 0) {
        if (means) means[0] = means[1] = 0.0;
        return 0;
    }
    if (!x || !scales || !stats) return 1;
    B = block_len(n, block);
    nb = (n + B - 1) / B;
    part = (long double *)malloc(nb * 2 * sizeof(long double));
    if (!part) return 4;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (b = 0; b < (long long)nb; ++b) {
        size_t lo = (size_t)b * B, hi = lo + B < n ? lo + B : n, i;
        float s = scales_given ? scales[b] : block_absmax(x, lo, hi);
        long double sum_abs = 0.0L, sum_rel = 0.0L;
        double count = 0.0, worst = 0.0;
        if (!scales_given) scales[b] = s;
        for (i = lo; i < hi; ++i) {
            float xn, q;
            double e;
            if (s == 0.0f)
                xn = x[i];
            else
                xn = x[i] / s;
            q = cb[nearest_code(cb, xn)] * s;
            e = fabs((double)q - (double)x[i]);
            sum_abs += (long double)e;
            if (x[i] != 0.0f) {
                double rel = e / fabs((double)x[i]); /* one binary64 division per term */
                sum_rel += (long double)rel;
                count += 1.0;
            }
            if (e > worst) worst = e;
        }
        part[2 * b] = sum_abs;
        part[2 * b + 1] = sum_rel;
        stats[4 * b] = (double)sum_abs;
        stats[4 * b + 1] = (double)sum_rel;
        stats[4 * b + 2] = count;
        stats[4 * b + 3] = worst;
    }
    if (means) {
        long double ta = 0.0L, tr = 0.0L;
        double tc = 0.0;
        for (b = 0; b < (long long)nb; ++b) {
            ta += part[2 * b];
            tr += part[2 * b + 1];
            tc += stats[4 * b + 2];
        }
        means[0] = (double)(ta / (long double)n);
        means[1] = tc > 0.0 ? (double)(tr / (long double)tc) : 0.0;
    }
    free(part);
    return 0;
}
