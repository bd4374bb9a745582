// dq8: the average-then-compress round for blocks of 513 .. 3072 elements
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

// Average-then-compress for blocks of up to 3072 elements: teams of W = 1, 2 or 3 wavefronts, a block per team
// (W x 1024 elements hold it), twelve wavefronts per workgroup and one workgroup per compute unit.
int launch_avg_short_team_tu(int cus, const uint32_t *tab, uint32_t search_words, bool has_remap, const uint8_t *const *codes,
                             const float *const *scales, int K, const float *local, size_t n, size_t block, float *scales_out,
                             uint8_t *codes_out, hipStream_t stream)
{
    const WorkerPtrs wp = gather(codes, scales, K);
    const size_t Bq = block_length(n, block);
    const int W = (int)((Bq + 1023) / 1024);
    const bool ragged = Bq != (size_t)W * 1024;
    const int teams = 12 / W;
    Plan p = make_plan(n, block, cus, 12, W, 12, kUnit);
    const uint32_t iters = (uint32_t)((p.n_units + p.n_teams - 1) / p.n_teams);
    // Iterations in which every team's current and next unit are whole aligned blocks.
    uint32_t steady = 0;
    bool aligned = !ragged && ((uintptr_t)codes_out & 3) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) aligned = aligned && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (aligned) {
        const size_t all_valid = (n / Bq) / p.n_teams;  // iterations in which every team has a whole unit
        if (all_valid >= 2) steady = (uint32_t)((all_valid - 1) & ~(size_t)1);
    }
    const size_t lds = ((size_t)search_words + 2 * teams * kWavesPerWg) * sizeof(uint32_t);
#define DQ8_SHORT(KT, RM, RG, WW)                                                                                          \
    hipLaunchKernelGGL((k_avg_team<KT, 1, true, 12 / WW, RM, RG, false, WW>), dim3(p.grid), dim3(kWave * 12), lds, stream, tab, \
                       wp, K, local, n, p.B, p.nb, p.n_units, p.n_teams, iters, steady, scales_out, codes_out)
#define DQ8_SHORT_RG(KT, RM, WW)       \
    if (ragged) {                      \
        DQ8_SHORT(KT, RM, true, WW);   \
    } else {                           \
        DQ8_SHORT(KT, RM, false, WW);  \
    }
#define DQ8_SHORT_W(KT, RM)                      \
    switch (W) {                                 \
    case 1: DQ8_SHORT_RG(KT, RM, 1) break;       \
    case 2: DQ8_SHORT_RG(KT, RM, 2) break;       \
    default: DQ8_SHORT_RG(KT, RM, 3) break;      \
    }
#define DQ8_SHORT_K(KT)              \
    if (has_remap) {        \
        DQ8_SHORT_W(KT, true)        \
    } else {                         \
        DQ8_SHORT_W(KT, false)       \
    }
    switch (K) {
    case 1: DQ8_SHORT_K(1) break;
    case 2: DQ8_SHORT_K(2) break;
    case 3: DQ8_SHORT_K(3) break;
    case 4: DQ8_SHORT_K(4) break;
    case 5: DQ8_SHORT_K(5) break;
    case 6: DQ8_SHORT_K(6) break;
    case 7: DQ8_SHORT_K(7) break;
    default: DQ8_SHORT_K(8) break;
    }
#undef DQ8_SHORT_K
#undef DQ8_SHORT_W
#undef DQ8_SHORT_RG
#undef DQ8_SHORT
    return after_launch_of("k_avg_team", stream);
}

}  // namespace dq8
