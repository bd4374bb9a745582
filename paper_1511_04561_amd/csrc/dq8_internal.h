// Entry points that exist only so that the host logic can be tested without a GPU.
// Not part of the public ABI (include/dq8.h); no compute kernel is launched by any of them.
#pragma once
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

// Host tables of a data type: values, thresholds and the flattened search table.
// Any output pointer may be NULL.
int dq8_internal_tables(int kind, float *cb256, float *thr127, uint32_t *lo_key, uint32_t *n_bucket, uint32_t *bucket,
                        uint32_t bucket_capacity);

// Ranks of a data type: *n_mag = number of distinct magnitudes; canon128[r] = the 7-bit field the
// encoder emits for the magnitude of rank r (ascending), entries from n_mag on repeat the last one.
// thr127 of dq8_internal_tables has n_mag - 1 thresholds followed by +inf.
int dq8_internal_ranks(int kind, uint32_t *n_mag, uint8_t *canon128);

// Unit sizes the launch logic derives from a block length: out4 = {elements per scale block, the unit for
// kernels whose units are pieces of a block when they start from `quads` quads per lane (a power of two up
// to 16) and `waves_per_cu` wavefronts per compute unit, the wavefronts per compute unit that go with it,
// the unit for kernels that hold a whole block}.
int dq8_internal_units(size_t n, size_t block, int quads, int waves_per_cu, size_t *out4);

// Workers per chunk that the decode-and-average kernel for arbitrary worker counts is launched with.
int dq8_internal_chunk_size(int K);

// Launch plan for n elements with the given block on a device with `cus` compute units,
// `waves_per_cu` resident wavefronts per compute unit, teams of `wpb` wavefronts and units of
// `unit` elements: out6 = {B, nb, units per block, units, teams, workgroups}.
int dq8_internal_plan(size_t n, size_t block, int cus, int waves_per_cu, int wpb, size_t unit, size_t *out6);

// Runs the kernels' code search (the same inline functions, compiled for the host) over every
// non-negative finite binary32 bit pattern and +inf, and compares it with the code of the rank that a count
// of the thresholds <= the value gives: the lookup for exact quotients on every value, the lookup for
// reciprocal products on every value that does not raise the proximity flag.  *mismatches = number of
// disagreements; *missed_near = number of values within the proximity window of a threshold that did not
// raise the flag.
int dq8_internal_check_search(int kind, uint64_t *mismatches, uint64_t *missed_near);

// The encoder's per-element arithmetic on the host (same inline functions): codes of x[0..n)
// for one given scale, through the reciprocal path with its exact fallback (use_reciprocal
// != 0) or through true divisions only.  *n_exact = elements that took a true division.
int dq8_internal_encode_host(int kind, const float *x, size_t n, float scale, int use_reciprocal, uint8_t *codes,
                             uint64_t *n_exact);

// Changes a launch-shape parameter (experiments only; results never depend on them).  Works only in a
// library compiled with -DDQ8_TUNABLE, and is not synchronised with calls in flight on other threads; the
// shipped library has constant launch shapes and returns DQ8_ERR_ARG here.
int dq8_internal_tune(const char *key, int value);

// Copies n floats device to device with the codec kernels' access pattern (bandwidth and
// counter calibration: exactly 4 bytes read and 4 written per element).
int dq8_internal_copy(float *dst, const float *src, size_t n, void *hip_stream);

// The current device as the runtime describes it: out5 = {compute units, peak engine clock in kHz, peak memory
// clock in kHz, memory bus width in bits, L2 cache bytes} (for the benchmark's report).
int dq8_internal_device_info(int *out5);

#ifdef __cplusplus
}
#endif
