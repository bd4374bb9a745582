// Host-side check of divide_by_count (csrc/dq8_arith.hpp), the three-instruction quotient that the
// average-then-compress kernels use for a number of terms that is not a power of two: compared with the
// correctly rounded division for every binary32 significand, both signs and every count 3 .. 33 that is not a
// power of two, in the binade of 1.0, and for every 64th significand in binades from the bottom to the top of the
// range the kernels allow (2^-100 .. 2^127).  The quotient only depends on the significand as long as nothing on
// the way leaves the normal range, which is what the other binades probe.  Also the scale test that guards it.
#include <cstdio>
#include <cstring>

#include "dq8_arith.hpp"

static float from_bits(uint32_t b)
{
    float f;
    std::memcpy(&f, &b, 4);
    return f;
}

static uint32_t bits_of(float f)
{
    uint32_t b;
    std::memcpy(&b, &f, 4);
    return b;
}

int main()
{
    long bad = 0, checked = 0;
    const int binades[] = {27, 28, 60, 126, 128, 200, 253, 254};  // biased exponents
    for (int c = 3; c <= 33; ++c) {
        if ((c & (c - 1)) == 0) continue;
        const float fk = (float)c;
        volatile float one = 1.0f;  // the reciprocal by a division at run time, as in the kernels
        const float rk = one / fk;
        auto check = [&](uint32_t bits) {
            const float a = from_bits(bits);
            volatile float want = a / fk;
            const float got = divide_by_count(a, fk, rk);
            ++checked;
            if (bits_of(got) != bits_of(want)) {
                if (bad++ < 10) std::printf("FAIL count %d a %a: got %a want %a\n", c, a, got, (float)want);
            }
        };
        for (uint32_t m = 0; m < (1u << 23); ++m) {
            check((127u << 23) | m);
            check((1u << 31) | (127u << 23) | m);
        }
        for (int e : binades)
            for (uint32_t m = 0; m < (1u << 23); m += 64) {
                check(((uint32_t)e << 23) | m | (m >> 17));
                check((1u << 31) | ((uint32_t)e << 23) | (m + 63));
            }
        check(0);  // +0 stays +0
    }
    // the guard: scale 0 or 2^-40 .. 2^100
    const struct { float s; bool ok; } scales[] = {{0.0f, true}, {0x1p-40f, true}, {0x1p100f, true}, {1.0f, true}, {1e-3f, true},
                                                   {0x1.fffffep-41f, false}, {0x1.000002p100f, false}, {1e-42f, false}, {3e38f, false}};
    for (const auto &t : scales)
        if (scale_keeps_sums_in_range(bits_of(t.s)) != t.ok) {
            std::printf("FAIL scale %a\n", t.s);
            ++bad;
        }
    if (scale_keeps_sums_in_range(0x7F800000u) || scale_keeps_sums_in_range(0x7FC00000u)) {
        std::printf("FAIL infinite or NaN scale accepted\n");
        ++bad;
    }
    std::printf("%ld quotients checked, %ld wrong\n", checked, bad);
    if (bad == 0) std::printf("division checks ok\n");
    return bad != 0;
}
