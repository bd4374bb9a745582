// dq8: the average-then-compress round for blocks of 4097 .. 16384 elements
// A translation unit of its own (see dq8_launch.hpp).  Built with the flags of dq8.hip.
#include <hip/hip_runtime.h>

#include <cstring>

#include "dq8.h"
#include "dq8_launch.hpp"
#include "dq8_plan.hpp"

#include "dq8_device.hpp"
#include "dq8_kernels_avg_encode.hpp"

namespace {

WorkerPtrs gather(const uint8_t *const *codes, const float *const *scales, int K)
{
    WorkerPtrs wp;
    std::memset(&wp, 0, sizeof(wp));
    for (int k = 0; k < K; ++k) {
        wp.codes[k] = codes[k];
        wp.scales[k] = scales[k];
    }
    return wp;
}

}  // namespace

namespace dq8 {

// Average-then-compress for blocks of 4097 .. 16384 elements: a workgroup per block.
int launch_avg_long_tu(int cus, const uint32_t *tab, uint32_t search_words, const uint8_t *const *codes,
                       const float *const *scales, int K, const float *local, size_t n, size_t block, float *scales_out,
                       uint8_t *codes_out, hipStream_t stream)
{
    const WorkerPtrs wp = gather(codes, scales, K);
    const size_t B = block_length(n, block);
    const size_t nb = (n + B - 1) / B;
    size_t teams = (size_t)cus * 2;  // two workgroups' tables fit the LDS of a compute unit
    if (teams > nb) teams = nb;
    const size_t lds = ((size_t)search_words + kLongSlots) * sizeof(uint32_t);
    // The register path needs 32-bit accesses to the codes and 128-bit ones to local at every block start.
    bool aligned = K >= 1 && (nb == 1 || (B & 3) == 0) && ((uintptr_t)codes_out & 3) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) aligned = aligned && ((uintptr_t)wp.codes[k] & 3) == 0;
#define DQ8_AVG_LONG(QL, NB, KT)                                                                                              \
    hipLaunchKernelGGL((k_avg_long<QL, NB, 2, KT>), dim3((unsigned)teams), dim3(kLongTeam), lds, stream, tab, wp, K, local, n, \
                       B, nb, (uint32_t)teams, (uint32_t)aligned, scales_out, codes_out)
    // Quads per lane that hold the block in a workgroup of 512 threads.  Up to eight workers have kernels of their
    // own, with one set of code words per worker where the registers allow (up to four quads per lane) and three or
    // four sets otherwise; more workers take the kernel that reads the count at run time, with four sets (it pads
    // the count to a multiple of four).
    const int ql = (int)((B + 4 * kLongTeam - 1) / (4 * kLongTeam));
#define DQ8_AVG_LONG_Q(NB_SHORT, NB_LONG, KT)            \
    switch (ql) {                                        \
    case 3: DQ8_AVG_LONG(3, NB_SHORT, KT); break;        \
    case 4: DQ8_AVG_LONG(4, NB_SHORT, KT); break;        \
    case 5: DQ8_AVG_LONG(5, NB_LONG, KT); break;         \
    case 6: DQ8_AVG_LONG(6, NB_LONG, KT); break;         \
    case 7: DQ8_AVG_LONG(7, NB_LONG, KT); break;         \
    default: DQ8_AVG_LONG(8, NB_LONG, KT); break;        \
    }
    switch (K) {
    case 1: DQ8_AVG_LONG_Q(2, 2, 1) break;
    case 2: DQ8_AVG_LONG_Q(2, 2, 2) break;
    case 3: DQ8_AVG_LONG_Q(3, 3, 3) break;
    case 4: DQ8_AVG_LONG_Q(4, 4, 4) break;
    case 5: DQ8_AVG_LONG_Q(5, 3, 5) break;
    case 6: DQ8_AVG_LONG_Q(6, 3, 6) break;
    case 7: DQ8_AVG_LONG_Q(7, 4, 7) break;
    case 8: DQ8_AVG_LONG_Q(8, 4, 8) break;
    default: DQ8_AVG_LONG_Q(4, 4, 0) break;
    }
#undef DQ8_AVG_LONG_Q
#undef DQ8_AVG_LONG
    return after_launch_of("k_avg_long", stream);
}

}  // namespace dq8
