// Geometry shared by the host's launch plans and the kernels: wavefront and unit sizes, and the unit
// (block, first element, length) that a unit index stands for.  Plain C++: compiles for the host alone
// (the launch plan and its tests) and for the device.
#pragma once
#include <cstddef>
#include <cstdint>

#if defined(__HIPCC__)
#define DQ8_HD __host__ __device__ __forceinline__
#else
#define DQ8_HD inline
#endif

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerWg = 4;
constexpr int kWg = kWave * kWavesPerWg;
constexpr int kUnit = 4096;                      // elements per unit
constexpr int kUnitQuads = kUnit / (4 * kWave);  // 16 quads per lane when one wave owns a unit

// The kernels for tensors back to back with one scale each (segments) walk the array in units of their own.
constexpr int kSegQ = 4;                     // quads per lane
constexpr int kSegUnit = kSegQ * 4 * kWave;  // 1024 elements per unit
constexpr int kSegWaves = 16;                // wavefronts per workgroup

// Geometry of unit u.  All values are wave-uniform.
struct Unit {
    size_t block;   // scale index
    size_t start;   // first element
    uint32_t len;   // 1..kUnit
};

// min(v, U) of a 64-bit count as 32 bits, U a power of two.  Written with a shift and a compare
// against zero so that it stays on the scalar unit: a 64-bit ordered compare of uniform values
// is done on the vector unit, and the compiler has been seen to drop the copy of such a result
// into the scalar condition bit when a branch on the same result follows, leaving a select
// that reads a stale condition (wrong unit lengths, accesses past the end of the arrays).
template <int U>
DQ8_HD uint32_t cap_to_unit(size_t v)
{
    static_assert(U > 0 && (U & (U - 1)) == 0, "unit sizes are powers of two");
    return (v >> __builtin_ctz(U)) != 0 ? (uint32_t)U : (uint32_t)v;
}

template <int U>
DQ8_HD Unit unit_of(size_t u, size_t n, size_t B, size_t nb, size_t upb)
{
    Unit r;
    size_t c;
    if (upb == 1) {
        r.block = u;
        c = 0;
    } else if (nb == 1) {
        r.block = 0;
        c = u;
    } else {
        r.block = u / upb;
        c = u - r.block * upb;
    }
    const size_t off = c * (size_t)U;
    r.start = r.block * B + off;
    const uint32_t in_block = cap_to_unit<U>(B - off), in_array = cap_to_unit<U>(n - r.start);
    r.len = in_block < in_array ? in_block : in_array;
    return r;
}

}  // namespace
