// Launch functions of the dq8 library that are compiled as translation units of their own (their kernels are the
// many variants of the average-then-compress round for shorter and for longer blocks; compiled separately they
// build in parallel with the rest).  Only plain types cross the boundary: every translation unit has its own copy
// of the kernel headers' internal types.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace dq8 {

// Error state after a launch, and the wait of DQ8_DEBUG=1; defined in dq8.hip.
int after_launch_of(const char *what, hipStream_t stream);

// `tab`: the data type's table image on the device, `search_words`: LDS words of its search table, `has_remap`: its
// code bytes can carry marks.  codes / scales: the K workers' device pointers (host arrays).
int launch_avg_short_team_tu(int cus, const uint32_t *tab, uint32_t search_words, bool has_remap, const uint8_t *const *codes,
                             const float *const *scales, int K, const float *local, size_t n, size_t block, float *scales_out,
                             uint8_t *codes_out, hipStream_t stream);
int launch_avg_long_tu(int cus, const uint32_t *tab, uint32_t search_words, const uint8_t *const *codes,
                       const float *const *scales, int K, const float *local, size_t n, size_t block, float *scales_out,
                       uint8_t *codes_out, hipStream_t stream);

}  // namespace dq8
