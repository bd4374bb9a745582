// Host-side construction of the per-type tables the kernels search.
//
// For each 8-bit data type of Sec. 3.1 of arXiv 1511.04561 the library keeps
//   cb[256]      the value of every code (bit 7 = sign, bits 6..0 = magnitude index),
//   thr[]        thr[j] = smallest binary32 number strictly above the real midpoint of the
//                distinct magnitudes of rank j and j+1, so that the rank of the nearest
//                magnitude to |xn|, with ties to the smaller one, is  #{ j : thr[j] <= |xn| },
//   bucket[]     the same search flattened into one lookup, see below.
//
// Sec. 3.2 of the paper searches a sorted table of the 128 positive values with a
// binary search; the bucket table replaces the seven dependent steps of that search by
// one lookup keyed on the top bits of |xn| plus one integer add.
//
// Bucket table.  a = bits(|xn|) clamped to [lo_bits, hi_bits] with
//   lo_bits = (lo_key << 16) + 0x8000,  hi_bits = (hi_key << 16) + 0x8000,
// the middles of two buckets that hold no threshold and lie below the first / above the
// last threshold (so clamping never changes the answer, and covers |xn| > 1, inf, NaN).
// key = a >> 16 (8 exponent bits + 7 mantissa bits).  The table is built from the thresholds
// moved down by W = kNearWindow binary32 steps, T' = T - W (see "Proximity" for why).  Every key
// range [key << 16, (key << 16) + 0xFFFF] contains at most one T' (checked when the table is
// built).  The entry is
//   S = (base << 16) + (0x10000 - t)
// where base = number of T' below the range and t = low 16 bits of the T' inside the range
// (t = 0x10000 when there is none).  Then
//   sum = S + (a & 0xFFFF),   sum >> 16 = #{ T' <= a }
// because the add carries into bit 16 exactly when the low bits reach t.
//
// Proximity.  The encoder first takes the quotient as x * fl(1/s), which can differ from the
// correctly rounded x / s by up to three binary32 steps, and has to notice when that may
// matter.  The low 16 bits of sum are (a - T') mod 2^16 in a bucket with a T' and a & 0xFFFF
// in one without, so
//   (sum & 0xFFFF) <= 2 W
// holds for every a in [T - W, T + W] (when T + W lies past the end of the bucket, the next
// bucket has no T' of its own - thresholds are more than a bucket + 2 W apart, see
// build_tables - and a is within 2 W of its start), and otherwise only for values within 2 W
// of the start of a bucket or, harmlessly, far below a T' at the end of theirs.  A product
// that does not raise this flag is more than W steps away from every threshold, so it lies
// on the same side of every T, and of every T', as the true quotient: its sum >> 16 is the
// rank of the true quotient.  Products that raise the flag are recomputed with a true
// division, and the exact quotient A is looked up as a = A - W (on the bit patterns):
// #{ T' <= A - W } = #{ T <= A }.
//
// Codes instead of ranks.  `base` is not the rank itself but the 7-bit code field of that rank
// (canon[rank]), so that sum >> 16 is the code.  For the tree and linear types the two are the
// same.  The mantissa type has fields of equal value, of which only the smallest is a code, so
// its codes are ascending with gaps: a carry must take canon[r] to canon[r + 1].  Wherever
// canon[r + 1] == canon[r] + 1 the carry does that by itself.  The only other step the scheme
// accepts is the mantissa type's: from a field 16 E + 15 to 16 (E + 1) + 2 (fields 16 (E + 1)
// and 16 (E + 1) + 1 repeat smaller values).  A bucket whose threshold is such a step gets bit
// 7 of its code byte set as a mark; the byte then reads 0x80 | (16 E + 15) below the threshold
// and 0x80 | 16 (E + 1) above it, and fix_marked_codes (dq8_device.hpp) turns these into
// 16 E + 15 and 16 (E + 1) + 2, four packed code bytes at a time.
//
// Proximity.  The low 16 bits of sum are (a - threshold) mod 2^16 in a bucket with a
// threshold and (a & 0xFFFF) in one without.  ((sum + W) & 0xFFFF) <= 2 W therefore holds
// whenever a is within W binary32 steps of a threshold (also of one just across a bucket
// edge, because thresholds are more than a bucket + 2 W apart, see build_tables) and
// otherwise only for values within W steps of a bucket edge.  The encoder uses this to
// decide when a quotient computed as x * (1/s) may differ from the correctly rounded x / s
// in a way that matters, and redoes those with a true division.
#pragma once
#include <cstdint>

namespace dq8 {

constexpr uint32_t kNearWindow = 4;  // proximity window W in binary32 steps
constexpr int kTableWords = 4352;   // device words reserved per data type
constexpr int kCbOff = 0;           // 256 words: cb as raw binary32
constexpr int kLoKeyOff = 256;      // 1 word
constexpr int kNBucketOff = 257;    // 1 word
constexpr int kHasMarksOff = 258;   // 1 word: non-zero when some buckets carry the mark for a step of 3 (see above)
constexpr int kBucketOff = 260;     // bucket entries, 16-byte aligned
constexpr int kBucketCapacity = kTableWords - kBucketOff;

struct Tables {
    float cb[256];
    // Distinct magnitudes in ascending order are ranked 0 .. n_mag - 1; thr[r] separates rank r
    // from rank r + 1 and canon[r] is the 7-bit magnitude field the encoder emits for rank r.
    // For the tree and linear types every field is its own rank (n_mag == 128, canon[r] == r).
    // The mantissa type has fields of equal value; the smallest field of a value is its code.
    uint32_t n_mag;
    uint8_t canon[128];
    bool has_marks;  // some buckets carry the mark: code bytes have to pass through fix_marked_codes
    float thr[127];  // n_mag - 1 entries used
    uint32_t lo_key;
    uint32_t n_bucket;
    uint32_t bucket[kBucketCapacity];
};

// Returns 0 on success, 2 for an unknown kind, 5 if the type does not fit the bucket scheme.
int build_tables(int kind, Tables *t);

// Packs t into the kTableWords-word device image.
void pack_tables(const Tables &t, uint32_t *words);

}  // namespace dq8
