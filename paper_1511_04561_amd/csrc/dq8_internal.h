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

// Launch plan for n elements with the given block on a device with `cus` compute units:
// out6 = {B, nb, units per block, units, wavefronts, workgroups}.
int dq8_internal_plan(size_t n, size_t block, int cus, size_t *out6);

// Runs the kernels' code search (the same inline function, compiled for the host) over every
// non-negative finite binary32 bit pattern and +inf, and compares it with a count of the
// thresholds that are <= the value.  *mismatches receives the number of disagreements.
int dq8_internal_check_search(int kind, uint64_t *mismatches);

// The kernels' code search on the host for an array of already normalised values.
int dq8_internal_search(int kind, const float *xn, size_t n, uint8_t *codes);

// Copies n floats device to device with the codec kernels' access pattern (bandwidth and
// counter calibration: exactly 4 bytes read and 4 written per element).
int dq8_internal_copy(float *dst, const float *src, size_t n, void *hip_stream);

#ifdef __cplusplus
}
#endif
