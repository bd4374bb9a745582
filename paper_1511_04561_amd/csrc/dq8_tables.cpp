// Host-side table construction for the dq8 kernels (see dq8_tables.hpp).
#include "dq8_tables.hpp"

#include <cmath>
#include <cstring>

namespace dq8 {
namespace {

uint32_t f2u(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}

float u2f(uint32_t u)
{
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// num / den rounded once to binary32 (nearest, ties to even), in integer arithmetic.
// Requires 0 <= num / den < 2 and a result that is zero or a normal number.
float ratio_to_f32(uint64_t num, uint64_t den)
{
    if (num == 0) return 0.0f;
    // scale so that q = floor(num * 2^sh / den) has exactly 25 significant bits
    int sh = 0;
    unsigned __int128 n = num;
    while (n / den < ((unsigned __int128)1 << 24)) {
        n <<= 1;
        ++sh;
    }
    unsigned __int128 q = n / den, r = n % den;
    uint32_t m = (uint32_t)(q >> 1);  // 24-bit significand candidate
    bool half = (q & 1) != 0, sticky = r != 0;
    if (half && (sticky || (m & 1))) ++m;
    // value = m * 2^-(sh-1); m == 2^24 after a carry is still exact in ldexp
    return std::ldexp((float)m, -(sh - 1));
}

uint64_t pow10u(int e)
{
    uint64_t p = 1;
    while (e-- > 0) p *= 10;
    return p;
}

// Magnitude j of each data type of Sec. 3.1 as an exact ratio num / den.
bool magnitude_ratio(int kind, int j, uint64_t *num, uint64_t *den)
{
    if (kind == 0) {  // dynamic tree: [n zeros][1][t tree bits]
        if (j == 0) {
            *num = 0;
            *den = 1;
            return true;
        }
        int flag = 6;  // bit position of the flag inside the 7-bit field
        while (!((j >> flag) & 1)) --flag;
        int t = flag, n = 6 - flag;
        uint64_t leaf = (uint64_t)j & ((1u << t) - 1);  // path through the bisection tree
        // middle of leaf `leaf` of 2^t equal pieces of (0.1, 1):  1/10 + 9/10 * (2 leaf + 1) / 2^(t+1)
        *num = (1ull << (t + 1)) + 9 * (2 * leaf + 1);
        *den = (1ull << (t + 1)) * 10 * pow10u(n);
        return true;
    }
    if (kind == 1) {  // linear quantisation on [0, 1]
        *num = (uint64_t)j;
        *den = 127;
        return true;
    }
    if (kind == 2) {  // static tree: 3 exponent bits, 4 tree bits; decade 10^(E-7)
        int E = j >> 4;
        uint64_t leaf = (uint64_t)(j & 15);
        *num = 32 + 9 * (2 * leaf + 1);
        *den = 32ull * 10 * pow10u(7 - E);
        return true;
    }
    if (kind == 3) {  // mantissa: 3 exponent bits, 4-bit integer mantissa counting tenths of the decade 10^(E-7)
        int E = j >> 4;
        *num = (uint64_t)(j & 15);
        *den = 10 * pow10u(7 - E);
        return true;
    }
    return false;
}

}  // namespace

int build_tables(int kind, Tables *t)
{
    for (int j = 0; j < 128; ++j) {
        uint64_t num, den;
        if (!magnitude_ratio(kind, j, &num, &den)) return 2;
        t->cb[j] = ratio_to_f32(num, den);
        t->cb[j + 128] = u2f(f2u(t->cb[j]) | 0x80000000u);
    }
    // Rank the distinct magnitudes (binary32 values of non-negative numbers order like their bit
    // patterns); of several fields with one value the smallest is the code.
    float mag[128];
    uint32_t n_mag = 0;
    t->has_marks = false;
    for (;;) {
        int best = -1;
        for (int j = 0; j < 128; ++j) {
            if (n_mag > 0 && !(f2u(t->cb[j]) > f2u(mag[n_mag - 1]))) continue;  // ranked already, or a repeat of it
            if (best < 0 || f2u(t->cb[j]) < f2u(t->cb[best])) best = j;         // strict: the smallest field wins
        }
        if (best < 0) break;
        mag[n_mag] = t->cb[best];
        t->canon[n_mag] = (uint8_t)best;
        ++n_mag;
    }
    for (uint32_t r = n_mag; r < 128; ++r) t->canon[r] = t->canon[n_mag - 1];
    t->n_mag = n_mag;
    if (n_mag < 2) return 5;
    const int n_thr = (int)n_mag - 1;
    for (int j = 0; j < 127; ++j) t->thr[j] = u2f(0x7F800000u);  // unused entries: never reached
    for (int j = 0; j < n_thr; ++j) {
        // the midpoint of two nearby binary32 numbers is exact in binary64
        double mid = ((double)mag[j] + (double)mag[j + 1]) * 0.5;
        float f = (float)mid;
        if ((double)f <= mid) f = std::nextafterf(f, 4.0f);
        t->thr[j] = f;  // smallest binary32 strictly above the midpoint
        if (j > 0 && !(t->thr[j - 1] < f)) return 5;
    }
    if (!(t->thr[n_thr - 1] < 2.0f)) return 5;
    // Neighbouring thresholds must be more than a bucket apart (plus the width of the
    // encoder's proximity window on both sides): then a bucket holds at most one threshold
    // and a threshold close to a bucket edge has a threshold-free neighbour bucket.
    for (int j = 1; j < n_thr; ++j)
        if (f2u(t->thr[j]) - f2u(t->thr[j - 1]) <= 0x10000u + 2 * kNearWindow) return 5;
    // the table is built from the thresholds moved down by the proximity window (see dq8_tables.hpp)
    uint32_t moved[127];
    for (int j = 0; j < n_thr; ++j) moved[j] = f2u(t->thr[j]) - kNearWindow;
    uint32_t lo_key = (moved[0] >> 16);
    if (lo_key == 0) return 5;
    lo_key -= 1;  // one bucket that lies entirely below the first threshold
    // one bucket entirely above the last threshold and its window
    const uint32_t hi_key = ((f2u(t->thr[n_thr - 1]) + kNearWindow) >> 16) + 1;
    uint32_t nb = hi_key - lo_key + 1;
    if (nb > (uint32_t)kBucketCapacity) return 5;
    t->lo_key = lo_key;
    t->n_bucket = nb;
    int j = 0;  // next threshold not yet passed
    for (uint32_t key = lo_key; key <= hi_key; ++key) {
        uint32_t first = key << 16, last = first | 0xFFFFu;
        uint32_t base = (uint32_t)j, tlow = 0x10000u;
        int inside = 0;
        while (j < n_thr && moved[j] <= last) {
            if (moved[j] < first) return 5;  // cannot happen: thresholds ascend
            tlow = moved[j] & 0xFFFFu;
            ++inside;
            ++j;
        }
        if (inside > 1) return 5;  // two thresholds in one bucket: scheme not applicable
        // the code field of rank `base`; the carry of a bucket with a threshold must lead to the code of the next rank
        uint32_t field = t->canon[base];
        if (inside == 1) {
            const uint32_t next = t->canon[base + 1];
            if (next == field + 3 && (field & 15u) == 15u) {
                field |= 0x80u;  // the mark: see fix_marked_codes
                t->has_marks = true;
            } else if (next != field + 1) {
                return 5;  // a step between codes that neither the carry nor the mark can make
            }
        }
        t->bucket[key - lo_key] = (field << 16) + (0x10000u - tlow);
    }
    if (j != n_thr) return 5;
    return 0;
}

void pack_tables(const Tables &t, uint32_t *words)
{
    std::memset(words, 0, sizeof(uint32_t) * kTableWords);
    for (int c = 0; c < 256; ++c) words[kCbOff + c] = f2u(t.cb[c]);
    words[kLoKeyOff] = t.lo_key;
    words[kNBucketOff] = t.n_bucket;
    words[kHasMarksOff] = t.has_marks ? 1u : 0u;
    for (uint32_t i = 0; i < t.n_bucket; ++i) words[kBucketOff + i] = t.bucket[i];
}

}  // namespace dq8
