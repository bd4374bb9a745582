// Host-side construction of the per-type tables the kernels search.
//
// For each 8-bit data type of Sec. 3.1 of arXiv 1511.04561 the library keeps
//   cb[256]      the value of every code (bit 7 = sign, bits 6..0 = magnitude index),
//   thr[127]     thr[j] = smallest binary32 number strictly above the real midpoint of
//                magnitudes j and j+1, so that the nearest magnitude to |xn| with ties to
//                the smaller one is  #{ j : thr[j] <= |xn| },
//   bucket[]     the same search flattened into one lookup, see below.
//
// Sec. 3.2 of the paper searches a sorted table of the 128 positive values with a
// binary search; the bucket table replaces the seven dependent steps of that search by
// one lookup keyed on the top bits of |xn| plus one integer add.
//
// Bucket table.  key = bits(|xn|) >> 16 (8 exponent bits + 7 mantissa bits), clamped to
// [lo_key, lo_key + n_bucket - 1].  Every key range [key << 16, (key << 16) + 0xFFFF]
// contains at most one threshold (checked when the table is built).  The entry is
//   S = (base << 16) + (0x10000 - t)
// where base = number of thresholds below the range and t = low 16 bits of the threshold
// inside the range (t = 0x10000 when there is none).  Then
//   magnitude index = (S + (bits(|xn|) & 0xFFFF)) >> 16
// because the add carries into bit 16 exactly when the low bits reach t.
#pragma once
#include <cstdint>

namespace dq8 {

constexpr int kTableWords = 4096;   // device words reserved per data type
constexpr int kCbOff = 0;           // 256 words: cb as raw binary32
constexpr int kLoKeyOff = 256;      // 1 word
constexpr int kNBucketOff = 257;    // 1 word
constexpr int kBucketOff = 260;     // bucket entries, 16-byte aligned

struct Tables {
    float cb[256];
    float thr[127];
    uint32_t lo_key;
    uint32_t n_bucket;
    uint32_t bucket[kTableWords - kBucketOff];
};

// Returns 0 on success, 2 for an unknown kind, 5 if the type does not fit the bucket scheme.
int build_tables(int kind, Tables *t);

// Packs t into the kTableWords-word device image.
void pack_tables(const Tables &t, uint32_t *words);

}  // namespace dq8
