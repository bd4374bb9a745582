/*
 * dq8 -- 8-bit approximation codec for fp32 gradients and activations on AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "8-Bit Approximations for Parallelism in Deep Learning"
 * (arXiv 1511.04561): fp32 values are normalised by the absolute maximum of their block,
 * replaced by the nearest entry of a 256-entry table (one sign bit + 128 sorted magnitudes)
 * and sent as one byte each; the receiver looks the byte up and multiplies by the maximum.
 *
 * Conventions shared by every call
 *   - All `x`, `codes`, `scales`, `out` pointers are DEVICE pointers owned by the caller,
 *     unless a parameter is explicitly marked host.  The library allocates no memory the
 *     caller sees and keeps only small immutable per-device tables.
 *   - `n` is the number of elements.  `block` is the number of consecutive elements that
 *     share one scale: block == 0 means one scale for the whole array (the paper's
 *     per-matrix maximum); a row-major matrix gets one scale per row with block == row
 *     length.  nb = ceil(n / block) scales are read or written; the last block may be short.
 *   - `hip_stream` is a hipStream_t passed as void*; NULL is the default stream.  Work is
 *     enqueued on that stream and the call returns without waiting for it.  The first call
 *     on a device uploads the tables of all data types with a blocking copy; call
 *     dq8_init() beforehand where that must not happen (e.g. before stream capture).
 *   - Every function returns DQ8_OK or an error code and never throws or aborts.  After an
 *     error dq8_last_error() describes it.  n == 0 is DQ8_OK and launches nothing.
 *   - Inputs must be finite.  With DQ8_SCALES_GIVEN every scale must be finite and >= 0 (a zero
 *     scale means "do not divide") and the quotient x / scale must be finite; the sign bit of a
 *     code is taken from x, which is the sign of the quotient only for such scales.
 *   - Any pointer alignment and any n / block are accepted.  The fast paths need
 *     16-byte aligned `x` / `out`, 4-byte aligned `codes`, and block % 4 == 0 (or a single
 *     block); anything else runs on slower paths with the same results.  Blocks of 4096
 *     elements are the fastest; other lengths come close (the units of work follow the block
 *     or, where a block need not be held, the position in the array; powers of two from 4 to
 *     128 elements have kernels that pack many blocks into a wavefront); other lengths below
 *     256 use a fraction of each wavefront in the calls that compress.
 *   - Results are deterministic and independent of launch configuration: codes and scales
 *     are exact functions of the input, and the average adds workers in index order.
 *   - Calls may be made from several threads at once; the library shares only immutable tables.
 *   - DQ8_DEBUG=1 in the environment (read once, at the first launch of the process) makes every
 *     call wait for the stream after each kernel it launches and check the device's error
 *     state, so that a failing kernel is reported by the call that launched it (status
 *     DQ8_ERR_DEVICE, text in dq8_last_error()).  Calls are then synchronous; do not use it on a
 *     stream that is being captured into a graph.
 *
 * Code layout: bit 7 of a code is the sign, bits 6..0 index the 128 magnitudes in
 * ascending order.  This is this library's own layout; the paper's figure of the bit
 * fields is not reproduced and no wire compatibility with other implementations is claimed.
 */
#ifndef DQ8_H
#define DQ8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DQ8_OK = 0,
    DQ8_ERR_NULL = 1,   /* a required pointer is NULL */
    DQ8_ERR_KIND = 2,   /* unknown data type */
    DQ8_ERR_ARG = 3,    /* bad K, overlapping buffers, size overflow */
    DQ8_ERR_DEVICE = 4  /* a HIP call failed; text in dq8_last_error() */
};

/* The 8-bit data types of Sec. 3.1. */
enum {
    DQ8_DYNAMIC_TREE = 0, /* dynamic exponent + bisection tree over (0.1, 1) */
    DQ8_LINEAR = 1,       /* linear quantisation, magnitudes j / 127 */
    DQ8_STATIC_TREE = 2,  /* 3-bit static exponent + 4-bit bisection tree */
    DQ8_MANTISSA = 3      /* 3-bit static exponent + 4-bit integer mantissa 0..15 */
};

/* dq8_encode flag: `scales` is an input computed elsewhere (e.g. by dq8_absmax). */
#define DQ8_SCALES_GIVEN 1u

/* Largest number of worker buffers dq8_decode_accumulate_avg accepts. */
#define DQ8_MAX_K 32

/*
 * The table of a data type (Sec. 3.1): cb256_host[c] is the value code c stands for when the
 * scale is 1.  HOST pointer to 256 floats, written by the call.  Entries 0..127 are the
 * magnitudes (ascending for the tree and linear types), entry c + 128 is the negation of
 * entry c (so entry 128 is -0.0f where entry 0 is 0).  Pure host computation, needs no device.
 *   dynamic tree: entry 0 is 0; an entry whose 7-bit index has n leading zeros, then a one,
 *     then t = 6 - n bits read as k, is (0.1 + 0.9 (k + 1/2) / 2^t) * 10^-n;
 *   linear: j / 127;
 *   static tree: index = 16 E + k, value (0.1 + 0.9 (k + 1/2) / 16) * 10^(E - 7);
 *   mantissa: index = 16 E + m, value m * 10^(E - 8): the decades of the static tree, counted
 *     in tenths.  Its entries are not ascending and several stand for one value (m = 0 of every
 *     decade is zero, m = 10 of a decade is m = 1 of the next, and entries above 1 exist:
 *     1.1 .. 1.5); the encoder emits the smallest index among those of the nearest value, so
 *     encode(decode(c)) is that smallest index, not always c.  A decade offset as in
 *     Sec. 3.1 is a scale: pass scales 10^offset with DQ8_SCALES_GIVEN instead of the absmax.
 * Each entry is the exact ratio rounded once to binary32.
 */
int dq8_codebook(int kind, float *cb256_host);

/*
 * Uploads the tables of every data type to the current device (blocking).  Optional: the
 * other calls do it on first use.  Safe to call repeatedly and from several threads.
 * Once the tables are on a device the other calls only launch kernels on the given stream (no
 * allocation, no memset, no copy, no synchronisation), so they can be recorded into a HIP graph:
 * call dq8_init() on the device before the capture starts.
 */
int dq8_init(void);

/*
 * Block-wise absolute maximum (Sec. 3.1, last paragraph: a matrix is normalised by its
 * absolute maximum).  scales[b] = max |x[i]| over block b, exact, +0 for an all-zero block.
 * x: n floats (read).  scales: nb floats (written).
 */
int dq8_absmax(const float *x, size_t n, size_t block, float *scales, void *hip_stream);

/*
 * Compression (Sec. 3.1 last paragraph, Sec. 3.2 first paragraph).  For every element of
 * block b: xn = x[i] / scales[b] rounded once to binary32 (not divided when the scale is 0),
 * then codes[i] = the code whose table value is nearest to xn in real arithmetic; a value
 * exactly half way between two magnitudes takes the smaller one; bit 7 is the sign bit of xn.
 * x: n floats (read).  codes: n bytes (written).  scales: nb floats, written with the block
 * maxima unless flags has DQ8_SCALES_GIVEN, in which case they are read.
 * `codes` and `scales` must not overlap `x`.
 * x is read once when a block has at most 16384 elements (a block is held in registers between
 * the maximum and the quantisation); longer blocks, block == 0 on a longer array included,
 * take a maximum pass and a quantisation pass: x is read twice.
 */
int dq8_encode(int kind, const float *x, size_t n, size_t block, float *scales, uint8_t *codes,
               unsigned flags, void *hip_stream);

/*
 * Decompression (Sec. 3.2 third paragraph, Sec. 3.1 last paragraph):
 * out[i] = table[codes[i]] * scales[b], one binary32 multiplication.
 * codes: n bytes (read).  scales: nb floats (read).  out: n floats (written), must not
 * overlap the inputs.
 */
int dq8_decode(int kind, const uint8_t *codes, const float *scales, size_t n, size_t block,
               float *out, void *hip_stream);

/*
 * The same three steps for a set of matrices of any sizes laid out back to back in one array, each normalised
 * by its own absolute maximum (Sec. 3.1, last paragraph: the maximum is taken per matrix), in one call for
 * the whole set instead of one call per matrix (a gradient set of many small tensors is otherwise bound by
 * the cost of the calls).
 * bounds: DEVICE array of n_seg + 1 element offsets (read), bounds[0] = 0 <= bounds[1] <= ... <=
 * bounds[n_seg] = n; segment i is elements [bounds[i], bounds[i + 1]) and has scale scales[i]; an empty
 * segment gets scale +0.  1 <= n_seg <= DQ8_MAX_SEGMENTS.  The results are those of dq8_absmax / dq8_encode /
 * dq8_decode with block == 0 on every segment by itself.  The offsets are read on the device only: entries
 * beyond n count as n, and offsets that do not ascend give meaningless values, but no access outside the n
 * elements of the arrays and the n_seg scales.  flags as in dq8_encode.  Arrays as in the calls above, with
 * n_seg scales; outputs must not overlap inputs or each other.
 */
#define DQ8_MAX_SEGMENTS 4095
int dq8_absmax_segments(const float *x, size_t n, const uint64_t *bounds, size_t n_seg, float *scales,
                        void *hip_stream);
int dq8_encode_segments(int kind, const float *x, size_t n, const uint64_t *bounds, size_t n_seg, float *scales,
                        uint8_t *codes, unsigned flags, void *hip_stream);
int dq8_decode_segments(int kind, const uint8_t *codes, const float *scales, size_t n, const uint64_t *bounds,
                        size_t n_seg, float *out, void *hip_stream);
/* The K-way average of dq8_decode_accumulate_avg (Sec. 2.1) with the same segments: scales[k][i] is worker k's scale of
 * segment i.  local: NULL, or the caller's own n floats as the first term of every sum (Sec. 3.4), divisor K + 1 and
 * K >= 0 then; 1 <= K <= DQ8_MAX_K otherwise.  codes, scales: HOST arrays of K device pointers, as there. */
int dq8_decode_accumulate_avg_segments(int kind, const uint8_t *const *codes, const float *const *scales, int K,
                                       const float *local, size_t n, const uint64_t *bounds, size_t n_seg, float *out,
                                       void *hip_stream);

/*
 * Decompress K workers' buffers and average them (Sec. 2.1: data parallelism averages the
 * exchanged gradients) in one pass:
 *   acc = +0;  for k = 0 .. K-1 in this order: acc = acc + table[codes[k][i]] * scales[k][b];
 *   out[i] = acc / K
 * with the product, each sum and the quotient rounded to binary32 separately (no fused
 * multiply-add).  `codes` and `scales` are HOST arrays of K device pointers, read before the
 * call returns; buffer k holds n bytes / nb floats.  1 <= K <= DQ8_MAX_K.
 * out: n floats (written), must not overlap any input.
 */
int dq8_decode_accumulate_avg(int kind, const uint8_t *const *codes, const float *const *scales,
                              int K, size_t n, size_t block, float *out, void *hip_stream);

/*
 * The same average with the caller's own 32-bit gradient as one more term (Sec. 3.4, MNIST
 * paragraph: incoming buffers are 8-bit, the local GPU's gradient stays in 32 bits):
 *   acc = +0;  acc = acc + local[i];  then the K workers in index order as above;
 *   out[i] = acc / (K + 1)
 * every operation rounded to binary32 on its own.  local: n floats (read, device).
 * 0 <= K <= DQ8_MAX_K (K == 0: the local values alone; `codes` / `scales` may then be NULL).
 * out: n floats (written), must not overlap any input.
 */
int dq8_decode_accumulate_avg_local(int kind, const uint8_t *const *codes, const float *const *scales,
                                    int K, const float *local, size_t n, size_t block, float *out,
                                    void *hip_stream);

/*
 * Second round of the gradient exchange (Appendix, cluster model: the gradients are sent once
 * raw and once accumulated): average the K received buffers -- with `local` as the first term
 * when it is not NULL, divisor K + 1 -- and compress the averages again, without an fp32 array
 * in between.  Results are identical to dq8_decode_accumulate_avg[_local] followed by
 * dq8_encode of its output with the same kind and block.
 * out_scales: nb floats (written), out_codes: n bytes (written); neither may overlap an input.
 * A scale block must fit the registers of one workgroup: block (or n when block == 0) <= 16384,
 * otherwise DQ8_ERR_ARG (use the two separate calls).  1 <= K <= DQ8_MAX_K, or 0 <= K with local.
 */
int dq8_decode_avg_encode(int kind, const uint8_t *const *codes, const float *const *scales, int K,
                          const float *local, size_t n, size_t block, float *out_scales,
                          uint8_t *out_codes, void *hip_stream);

/*
 * Approximation error of a data type on a sample (Sec. 3.4, first paragraph, and Table 2: mean
 * absolute and mean relative error of compress-then-decompress; the tree and linear types
 * normalise by the absolute maximum, the static-exponent types may be given a decade as scale).
 * x: DEVICE, n floats, finite.  scales: DEVICE, ceil(n / block) floats; written with the block
 * maxima first (as dq8_encode does) unless flags has DQ8_SCALES_GIVEN, then read only.
 * stats: DEVICE, 4 doubles per block, written: with q = fl32(cb[code] * s) and
 * e = |(double) q - (double) x| (both roundings as written: one binary64 subtraction, one
 * correctly rounded binary64 division),
 *   stats[4 b + 0] = sum of e over block b
 *   stats[4 b + 1] = sum of e / |x| over the elements of the block with x != 0
 *   stats[4 b + 2] = number of elements with x != 0 (zeros have no relative error; divide by this)
 *   stats[4 b + 3] = largest e of the block.
 * means: DEVICE, 2 doubles, or NULL: means[0] = (sum of e over the array) / n, means[1] = (sum of
 * relative errors) / (number of non-zero x), 0 when all x are zero.
 * The count and the maximum are exact.  The sums are binary64 sums of non-negative terms whose
 * order is not fixed: they are within (terms) * 2^-52 (relative) of the real sums and may differ
 * in the last bits between calls.  stats and means 8-byte aligned; no buffer may overlap another.
 * n == 0 writes nothing.  Asynchronous on the stream like the other calls.
 */
int dq8_error_stats(int kind, const float *x, size_t n, size_t block, float *scales, unsigned flags, double *stats,
                    double *means, void *hip_stream);

/*
 * Single-node speed-up model (Appendix, "A theoretical single node model for 4 GPUs"): the
 * convolutional part runs data-parallel at one GPU's speed, the fully connected part runs
 * model-parallel over `sub_batches` passes of `parallel_fc_ms` each, and communication that
 * cannot be hidden under computation is added as penalties:
 *   *speedup = n_gpus * total_ms /
 *              ((total_ms - fc_ms) + conv_penalty_ms + sub_batches * parallel_fc_ms + fc_penalty_ms)
 * Pure host arithmetic in double precision; all pointers are HOST pointers.  DQ8_ERR_ARG when
 * n_gpus < 1, sub_batches < 0, a time is negative or not finite, fc_ms > total_ms or the
 * denominator is not positive.
 */
int dq8_model_speedup(int n_gpus, double total_ms, double fc_ms, double conv_penalty_ms, int sub_batches,
                      double parallel_fc_ms, double fc_penalty_ms, double *speedup);

/*
 * The penalty term of that model: *penalty_ms = sum over i of max(transfer_ms[i] - compute_ms[i], 0),
 * the part of each transfer that the computation it overlaps with does not cover (compute 0 for a
 * transfer that overlaps with nothing).  HOST arrays of `count` doubles; count == 0 gives 0.
 */
int dq8_model_penalty(const double *transfer_ms, const double *compute_ms, size_t count, double *penalty_ms);

/* Text of the calling thread's most recent error ("" if none).  Static storage, never NULL. */
const char *dq8_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DQ8_H */
