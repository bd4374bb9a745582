// Arithmetic that the kernels share with the host-side checks of it.  Plain C++: compiles for the host alone
// and for the device.
#pragma once
#include <cstdint>

#include "dq8_units.hpp"

namespace {

// fl(a / count) for a small whole count (3 .. 33, not a power of two) without the division's instruction
// sequence.  rk = fl(1 / count), correctly rounded.  q0 = fl(a * rk) is within two steps of the quotient, its
// remainder a - q0 * count is a small multiple of q0's last place and comes out of one fused multiply-add
// exactly, and q0 + remainder * rk, rounded once by a second one, is the correctly rounded quotient: checked on
// the host for every binary32 significand and every such count.  Holds for a = +0 and for 2^-100 <= |a| <= 2^127
// (nothing on the way leaves the normal range except the remainder, which stays a whole number of 2^-149);
// not for -0, infinities or NaN.  Three instructions per element instead of ten.
DQ8_HD float divide_by_count(float a, float count, float rk)
{
    const float q0 = a * rk;
    const float rem = __builtin_fmaf(-q0, count, a);
    return __builtin_fmaf(rem, rk, q0);
}

// Whether a worker's block scale (its bit pattern; scales are finite and not negative) keeps every term of the
// ordered sum, and with them every partial sum, at 0 or inside the range that divide_by_count needs: a term is a
// table value (0 or 2^-27 .. 1.5 in magnitude) times the scale, and every partial sum is a whole number of the
// smallest term's last place.  Scale 0 or 2^-40 .. 2^100.
constexpr uint32_t kSafeScaleLo = (127u - 40u) << 23, kSafeScaleHi = (127u + 100u) << 23;
DQ8_HD bool scale_keeps_sums_in_range(uint32_t bits) { return bits == 0 || bits - kSafeScaleLo <= kSafeScaleHi - kSafeScaleLo; }

}  // namespace
