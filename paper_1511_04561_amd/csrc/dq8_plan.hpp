// Host-side launch planning of the dq8 library: how an array with its scale blocks is cut into units and how
// many wavefronts, teams and workgroups walk them.  Plain C++ (no HIP), so that it can be compiled and checked
// on its own; dq8.hip includes it.
#pragma once
#include <cstddef>
#include <cstdint>

#include "dq8.h"
#include "dq8_units.hpp"

namespace {

// Elements per scale block: `block` as the caller passed it, the whole array for 0 or a longer block.
inline size_t block_length(size_t n, size_t block) { return (block == 0 || block > n) ? n : block; }

// Unit for the kernels in which units are pieces of a block: starting from *quads per lane, the largest
// power of two of them whose unit (quads * 256 elements) is no longer than a block, at least one; every
// halving doubles *waves_per_cu (up to 32) so that the bytes in flight per compute unit stay the same.
inline void fit_unit_to_block(size_t block_len, int *quads, int *waves_per_cu)
{
    while (*quads > 1 && (size_t)*quads * 4 * kWave > block_len) {
        *quads >>= 1;
        *waves_per_cu = *waves_per_cu * 2 > 32 ? 32 : *waves_per_cu * 2;
    }
}

// Workers per chunk for the decode-and-average kernel that takes any number of workers a chunk at a time: the
// size from 3 to 8 with the fewest empty places in the last chunk (an empty place repeats a load), the largest
// such size; fewer than 3 workers are one chunk; K = 0 (the local term alone) has no chunks at all.
inline int chunk_size(int K)
{
    if (K < 3) return K < 1 ? 1 : K;
    int best = 3;
    for (int c = 3, waste = DQ8_MAX_K; c <= 8; ++c) {
        const int w = (K + c - 1) / c * c - K;
        if (w <= waste) {
            waste = w;
            best = c;
        }
    }
    return best;
}

// Unit for the kernels that hold a whole block in registers: the smallest power of two of elements
// between 256 and 4096 that holds a block (4096 for longer blocks).
inline size_t holding_unit(size_t block_len)
{
    size_t unit = 256;
    while (unit < block_len && unit < (size_t)kUnit) unit <<= 1;
    return unit;
}

// The longest block that dq8_encode holds in a team's registers (maximum and quantisation from one read of x).
constexpr size_t kLongestHeldBlock = 16384;

// Elements per unit for compression: the smallest power of two that holds a block, up to 4096 when the scales
// are given and up to 16384 when the kernel computes them.
inline size_t encode_unit(size_t block_len, bool fused)
{
    if (fused && block_len > (size_t)kUnit && block_len <= kLongestHeldBlock) return block_len <= 8192 ? 8192 : 16384;
    return holding_unit(block_len);
}

struct Plan {
    size_t B, nb, upb, n_units, n_teams;
    unsigned grid;
};

// Units, and a grid in which every team (wpb wavefronts) walks the same number of them.
inline Plan make_plan(size_t n, size_t block, int cus, int waves_per_cu, int wpb, int waves_per_wg = kWavesPerWg,
               size_t unit = kUnit)
{
    Plan p;
    p.B = block_length(n, block);
    p.nb = (n + p.B - 1) / p.B;
    p.upb = (p.B + unit - 1) / unit;
    if (p.nb == 1) {
        p.n_units = (n + unit - 1) / unit;
    } else {
        size_t last = n - (p.nb - 1) * p.B;  // the last block may be short
        p.n_units = (p.nb - 1) * p.upb + (last + unit - 1) / unit;
    }
    size_t max_teams = (size_t)cus * (size_t)waves_per_cu / (size_t)wpb;
    if (max_teams < 1) max_teams = 1;
    size_t per_team = (p.n_units + max_teams - 1) / max_teams;
    size_t teams = (p.n_units + per_team - 1) / per_team;
    size_t teams_per_wg = (size_t)waves_per_wg / wpb;
    size_t grid = (teams + teams_per_wg - 1) / teams_per_wg;
    p.grid = (unsigned)grid;
    p.n_teams = grid * teams_per_wg;
    return p;
}

// ---- blocks of 4 .. 128 elements (powers of two): many blocks per 1024-element unit of a wavefront

constexpr int kSmallQ = 4;                          // quads per lane
constexpr size_t kSmallUnit = kSmallQ * 4 * kWave;  // 1024 elements

// Quads per block for those kernels, 0 when the block length does not qualify.  Blocks of 256 to 1024
// elements (one, two or four whole rows of a unit) qualify in the kernels that have to hold a block, up to
// the length from which the general kernel for that call is at least as fast: `longest`.
inline int small_block_lanes(size_t n, size_t block_len, size_t longest = 128)
{
    if (block_len < 4 || block_len > longest || (block_len & (block_len - 1)) != 0 || block_len >= n) return 0;
    return (int)(block_len / 4);
}

struct SmallPlan {
    size_t n_units = 0, n_waves = 0, done = 0;  // whole units, wavefronts in the grid, elements they cover
    unsigned grid = 0;
};

// Whole leading units of the array on `waves_per_cu` wavefronts per compute unit, `wpw` per workgroup.
inline SmallPlan make_small_plan(size_t n, int cus, int waves_per_cu, int wpw)
{
    SmallPlan p;
    p.n_units = n / kSmallUnit;
    if (p.n_units == 0) return p;
    size_t waves = (size_t)cus * (size_t)waves_per_cu;
    const size_t per = (p.n_units + waves - 1) / waves;
    waves = (p.n_units + per - 1) / per;
    p.grid = (unsigned)((waves + wpw - 1) / wpw);
    p.n_waves = (size_t)p.grid * wpw;
    p.done = p.n_units * kSmallUnit;
    return p;
}

// ---- tensors back to back, one scale each

struct SegPlan {
    size_t n_units, n_items, n_waves, lds;
    uint32_t group;
    unsigned grid;
};

// Units of kSegUnit elements on up to `waves_per_cu` wavefronts per compute unit, kSegWaves per workgroup.
// grouped (the maxima): an item of work is four units when a workgroup per compute unit still gets two items or more
// per wavefront, else one unit (short arrays: as many wavefronts as there are units).
inline SegPlan make_segment_plan(int cus, size_t n, size_t n_seg, int waves_per_cu, bool grouped = false)
{
    SegPlan p;
    p.n_units = (n + kSegUnit - 1) / kSegUnit;
    size_t waves = (size_t)cus * (size_t)waves_per_cu;
    p.group = grouped && p.n_units >= (size_t)cus * kSegWaves * 8 ? 4u : 1u;
    if (p.group == 4) waves = (size_t)cus * kSegWaves;
    p.n_items = (p.n_units + p.group - 1) / p.group;
    if (waves > p.n_items) waves = p.n_items;
    p.grid = (unsigned)((waves + kSegWaves - 1) / kSegWaves);
    p.n_waves = (size_t)p.grid * kSegWaves;
    p.lds = (n_seg + 1) * sizeof(uint64_t);
    return p;
}

}  // namespace
