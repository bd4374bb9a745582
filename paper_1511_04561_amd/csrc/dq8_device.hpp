// Device-side building blocks of the dq8 kernels for gfx950: constants, memory access policies,
// wavefront reductions, unit geometry, the encoder's code search and the decoder's lookup table.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "dq8.h"
#include "dq8_tables.hpp"
#include "dq8_units.hpp"
#include "dq8_arith.hpp"

namespace {

using dq8::kBucketOff;
using dq8::kHasMarksOff;
using dq8::kCbOff;
using dq8::kLoKeyOff;
using dq8::kNBucketOff;
using dq8::kNearWindow;
using dq8::kTableWords;

constexpr int kKinds = 4;
constexpr int kLutCopies = 64;                   // one copy of the decode table per lane
constexpr int kTeamSlots = 8;                    // LDS words for the cross-wave maximum (2 phases x 4 waves)

typedef float v4f __attribute__((ext_vector_type(4)));

// Tables of the data types, one image per device (each GPU holds its own copy).
__device__ __align__(256) uint32_t g_tables[kKinds][kTableWords];

struct WorkerPtrs {
    const uint8_t *codes[DQ8_MAX_K];
    const float *scales[DQ8_MAX_K];
};

// Streaming accesses: every byte is touched once, so loads and stores carry cache-policy
// bits that keep them from displacing each other in the caches.  NT is the policy:
//   0  plain loads and stores;
//   1  non-temporal loads and stores (the nt bit);
//   2  non-temporal loads; 128-bit stores with nt plus system scope (sc0 sc1), i.e. streamed
//      through every cache level; 32-bit stores as in policy 1.
// The scope bits only strengthen coherence, so every policy gives the same memory contents.
//
// The compiler has no way to ask for "sc0 sc1 nt" on an ordinary store (a volatile store gets
// sc0 sc1 but is also made to wait for completion), so policy 2 writes the instruction out.
// A 128-bit store keeps reading its data registers for two cycles after issue; the compiler
// cannot see that this statement is such a store, so the two wait states it would otherwise
// insert before the next vector write to those registers are part of the statement.
template <int NT, typename T>
__device__ __forceinline__ T ldg(const T *p)
{
    if constexpr (NT != 0)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

template <int NT, typename T>
__device__ __forceinline__ void stg(T *p, T v)
{
    if constexpr (NT == 0)
        *p = v;
    else if constexpr (NT == 2 && sizeof(T) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    else
        __builtin_nontemporal_store(v, p);
}

// Maximum over the 64 lanes, returned in a scalar register.  Six data-parallel-primitive steps
// on the vector unit (no LDS traffic): exchange inside quads, mirror inside half rows and rows
// of 16 lanes, then carry lane 15 of a row into the next row and lane 31 into the upper half;
// lane 63 ends up with the maximum of all lanes.  A step leaves lanes it does not write at
// their own value, which is the identity of max.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t max_dpp(uint32_t v)
{
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xF, false);
    return o > v ? o : v;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max_dpp<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
    v = max_dpp<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
    v = max_dpp<0x141, 0xF>(v);  // row_half_mirror
    v = max_dpp<0x140, 0xF>(v);  // row_mirror
    v = max_dpp<0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
    v = max_dpp<0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

__host__ __device__ __forceinline__ uint32_t f2u(float f)
{
    uint32_t u;
    __builtin_memcpy(&u, &f, 4);
    return u;
}

__host__ __device__ __forceinline__ float u2f(uint32_t u)
{
    float f;
    __builtin_memcpy(&f, &u, 4);
    return f;
}

__device__ __forceinline__ uint32_t abs_bits(float f) { return f2u(f) & 0x7FFFFFFFu; }

// Running maximum of |v|.  Exact for finite inputs, subnormals included.
__device__ __forceinline__ float max4_abs(v4f v, float m)
{
    float a = __builtin_fmaxf(__builtin_fabsf(v.x), __builtin_fabsf(v.y));
    float b = __builtin_fmaxf(__builtin_fabsf(v.z), __builtin_fabsf(v.w));
    return __builtin_fmaxf(m, __builtin_fmaxf(a, b));
}

// Search state for the encoder (see dq8_tables.hpp): bucket table plus the clamp range, and whether
// code bytes of this data type can carry the mark of a step of 3 between codes.
struct Search {
    const uint32_t *bucket;  // LDS on the device
    bool marks;              // code bytes have to pass through fix_marked_codes
    uint32_t lo_key;         // key of the first bucket
    float lo_f, hi_f;        // clamp range as binary32 values (bit patterns lo_bits, hi_bits)
};

__host__ __device__ __forceinline__ Search make_search(const uint32_t *bucket, uint32_t lo_key, uint32_t n_bucket,
                                                       bool marks = false)
{
    Search s;
    s.bucket = bucket;
    s.marks = marks;
    s.lo_key = lo_key;
    s.lo_f = u2f((lo_key << 16) + 0x8000u);
    s.hi_f = u2f(((lo_key + n_bucket - 1) << 16) + 0x8000u);
    return s;
}

// Lookup of a = bits(|xn|) clamped into the table's range.  Byte 2 of the result (bits 16..23) is the code field
// of rank #{ T - W <= a } (T the thresholds, W = kNearWindow; possibly marked, see fix_marked_codes); its low half
// is small (is_near) whenever a lies within W steps of a threshold.  Non-negative binary32 values order like their
// bit patterns, so the clamp is done on the value.  SHIFT = W looks up a - W instead: the exact rank #{ T <= a }.
template <uint32_t SHIFT>
__host__ __device__ __forceinline__ uint32_t table_sum(const Search &s, float xn)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const float c = __builtin_amdgcn_fmed3f(__builtin_fabsf(xn), s.lo_f, s.hi_f);
#else
    float c = __builtin_fabsf(xn);
    c = c >= s.lo_f ? c : s.lo_f;  // also takes NaN to the low end; inputs are finite anyway
    c = c <= s.hi_f ? c : s.hi_f;
#endif
    const uint32_t a = f2u(c) - SHIFT;  // the clamp range is the middle of a bucket: a - W stays inside the table
    return s.bucket[(a >> 16) - s.lo_key] + (a & 0xFFFFu);
}

// For a quotient taken as x * fl(1 / s): right unless is_near(sum) says that a threshold is within W steps.
__host__ __device__ __forceinline__ uint32_t search_sum(const Search &s, float xn) { return table_sum<0>(s, xn); }

// For a correctly rounded quotient: always right.
__host__ __device__ __forceinline__ uint32_t search_sum_exact(const Search &s, float xn) { return table_sum<kNearWindow>(s, xn); }

// Distance measure of a search_sum result: values up to 2 W mean "within W steps of a threshold (or just past
// the start of a bucket)".
__host__ __device__ __forceinline__ uint32_t near_key(uint32_t sum) { return sum & 0xFFFFu; }

// Up to four code bytes in one word.  A byte with bit 7 set comes from a bucket whose threshold separates code
// 16 E + 15 from code 16 (E + 1) + 2 (the two fields in between repeat smaller values and are never emitted):
// its low seven bits are 16 E + 15 when the value lies below the threshold and 16 (E + 1) when the carry of the
// search has happened.  Clearing the mark and setting bit 1 of the bytes whose bit 0 is clear gives the codes.
// Bytes without the mark pass unchanged.
__host__ __device__ __forceinline__ uint32_t fix_marked_codes(uint32_t m)
{
    const uint32_t marked = (m >> 7) & 0x01010101u;  // bit 0 of every marked byte
    const uint32_t carried = marked & ~m;            // ... whose own bit 0 is clear
    return (m & 0x7F7F7F7Fu) | (carried << 1);
}

// Code = code field (byte 2 of sum), bit 7 = sign bit of the input (the divisor is not negative).
__host__ __device__ __forceinline__ uint32_t code_of(const Search &s, uint32_t sum, float x)
{
    uint32_t m = (sum >> 16) & 0xFFu;
    if (s.marks) m = fix_marked_codes(m);
    return m | ((f2u(x) >> 24) & 0x80u);
}

__host__ __device__ __forceinline__ uint32_t code_exact(const Search &s, float x, float d) { return code_of(s, search_sum_exact(s, x / d), x); }

// Four codes in one word: byte i = code field of sum i (its byte 2) with the sign bit of
// x i (top bit of its byte 3).  v_perm_b32 gathers the bytes: selector byte 0..3 picks a byte
// of the second operand, 4..7 of the first, 0x0C gives zero.
__device__ __forceinline__ uint32_t pack_codes(const Search &sr, uint32_t s0, uint32_t s1, uint32_t s2, uint32_t s3, v4f v)
{
    const uint32_t m01 = __builtin_amdgcn_perm(s1, s0, 0x0C0C0602u);
    const uint32_t m23 = __builtin_amdgcn_perm(s3, s2, 0x06020C0Cu);
    const uint32_t g01 = __builtin_amdgcn_perm(f2u(v.y), f2u(v.x), 0x0C0C0703u);
    const uint32_t g23 = __builtin_amdgcn_perm(f2u(v.w), f2u(v.z), 0x07030C0Cu);
    uint32_t m = m01 | m23;
    if (sr.marks) m = fix_marked_codes(m);
    return ((g01 | g23) & 0x80808080u) | m;
}

// A scale qualifies for the reciprocal path when 1/d and every product x * (1/d) that can
// reach a threshold are normal numbers: 2^-98 <= d <= 2^100.  (The lower end leaves room for two things: a
// reciprocal that is scaled by up to 2^-5 more, and values below the normal range, |x| < 2^-126, whose quotient
// is then below 2^-28, under the smallest threshold of every data type by a quarter of its value.)
__host__ __device__ __forceinline__ bool reciprocal_ok(float d)
{
    uint32_t b = f2u(d);
    return b >= 0x0E800000u && b <= 0x71800000u;
}

// Four codes packed into one word.  With `recip` the quotients are first taken as x * r with
// r = fl(1/d): that differs from the correctly rounded x / d by at most 3 binary32 steps, so
// the code is already right unless the product lies within kNearWindow steps of a threshold;
// if any lane of the wavefront sees such a value the quad is redone with true divisions.
template <bool FASTDIV>
__device__ __forceinline__ uint32_t encode_quad(const Search &sr, v4f v, float d, float r, bool recip)
{
    if (FASTDIV && recip) {
        const uint32_t s0 = search_sum(sr, v.x * r), s1 = search_sum(sr, v.y * r);
        const uint32_t s2 = search_sum(sr, v.z * r), s3 = search_sum(sr, v.w * r);
        uint32_t k0 = near_key(s0), k1 = near_key(s1), k2 = near_key(s2), k3 = near_key(s3);
        k0 = k0 < k1 ? k0 : k1;
        k2 = k2 < k3 ? k2 : k3;
        k0 = k0 < k2 ? k0 : k2;
        if (__builtin_amdgcn_ballot_w64(k0 <= 2 * kNearWindow) == 0) return pack_codes(sr, s0, s1, s2, s3, v);
    }
    return pack_codes(sr, search_sum_exact(sr, v.x / d), search_sum_exact(sr, v.y / d), search_sum_exact(sr, v.z / d), search_sum_exact(sr, v.w / d), v);
}

// Q quads at once: all 4 Q table lookups of the reciprocal path are issued before the first result is
// used, so their latencies overlap.  One test covers all of them; only when some lane of the wavefront has a
// value next to a threshold (about one group in five) is each quad checked, and redone with true divisions, on
// its own.
// The values to compress are v * pre, with pre = 1 or a power of two 2^-k, k <= 5, that the caller has not
// multiplied in: the products v * pre are exact scalings for every result in the normal range, so
// v * (pre * r) is the same number as (v * pre) * r and one multiplication per element is saved; results below
// the normal range lie under every threshold (see reciprocal_ok) and get rank 0 either way.  Sign bits come
// from v, which has the sign of v * pre.
template <bool FASTDIV, int Q>
__device__ __forceinline__ void encode_quads(const Search &sr, const v4f (&v)[Q], float pre, float d, float r, bool recip,
                                             uint32_t (&cw)[Q])
{
    if (FASTDIV && recip) {
        const float rp = r * pre;  // exact: r is within [2^-100, 2^98]
        uint32_t s[Q][4], k[Q];
#pragma unroll
        for (int it = 0; it < Q; ++it) {
            s[it][0] = search_sum(sr, v[it].x * rp);
            s[it][1] = search_sum(sr, v[it].y * rp);
            s[it][2] = search_sum(sr, v[it].z * rp);
            s[it][3] = search_sum(sr, v[it].w * rp);
        }
        uint32_t all = 0xFFFFu;
#pragma unroll
        for (int it = 0; it < Q; ++it) {
            const uint32_t k01 = near_key(s[it][0]) < near_key(s[it][1]) ? near_key(s[it][0]) : near_key(s[it][1]);
            const uint32_t k23 = near_key(s[it][2]) < near_key(s[it][3]) ? near_key(s[it][2]) : near_key(s[it][3]);
            k[it] = k01 < k23 ? k01 : k23;
            all = all < k[it] ? all : k[it];
        }
        if (__builtin_amdgcn_ballot_w64(all <= 2 * kNearWindow) != 0) {
#pragma unroll
            for (int it = 0; it < Q; ++it) {
                if (__builtin_amdgcn_ballot_w64(k[it] <= 2 * kNearWindow) != 0) {
                    s[it][0] = search_sum_exact(sr, (v[it].x * pre) / d);
                    s[it][1] = search_sum_exact(sr, (v[it].y * pre) / d);
                    s[it][2] = search_sum_exact(sr, (v[it].z * pre) / d);
                    s[it][3] = search_sum_exact(sr, (v[it].w * pre) / d);
                }
            }
        }
#pragma unroll
        for (int it = 0; it < Q; ++it) cw[it] = pack_codes(sr, s[it][0], s[it][1], s[it][2], s[it][3], v[it]);
    } else {
#pragma unroll
        for (int it = 0; it < Q; ++it) {
            const v4f m = {v[it].x * pre, v[it].y * pre, v[it].z * pre, v[it].w * pre};
            cw[it] = encode_quad<false>(sr, m, d, r, recip);
        }
    }
}

template <bool FASTDIV, int Q>
__device__ __forceinline__ void encode_quads(const Search &sr, const v4f (&v)[Q], float d, float r, bool recip, uint32_t (&cw)[Q])
{
    encode_quads<FASTDIV, Q>(sr, v, 1.0f, d, r, recip, cw);
}

// The sums of `terms` terms become means, and their largest magnitude is returned.  When the number of terms is a
// power of two the division is a scaling by rk = 1 / terms, which commutes with the maximum and with everything
// the compression does (see encode_quads): the sums are left as they are, *pre = rk, and the maximum is scaled
// once (rounding is monotonic, so the scaled maximum is the maximum of the scaled values, also below the normal
// range).  Otherwise every sum is divided and *pre = 1: with the three instructions of divide_by_count when the
// caller knows that the sums are 0 or in its range (`in_range`: no local term and every worker's scale for the block
// passes scale_keeps_sums_in_range), with the division proper when not.
// LEAVE_SCALING = false: the sums are multiplied by rk here and *pre = 1 (a kernel that is short of registers: a *pre
// that is not a constant costs the compression about thirty of them).  One test per unit either way, not one per element.
template <int Q, bool LEAVE_SCALING = true>
__device__ __forceinline__ float means_for_compression(v4f (&acc)[Q], bool pow2, float rk, float fk, float *pre, bool in_range = false)
{
    float fm = 0.0f;
    if (pow2 && LEAVE_SCALING) {
#pragma unroll
        for (int j = 0; j < Q; ++j) fm = max4_abs(acc[j], fm);
        *pre = rk;
        return fm * rk;
    }
    *pre = 1.0f;
    if (pow2) {
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            acc[j] = v4f{acc[j].x * rk, acc[j].y * rk, acc[j].z * rk, acc[j].w * rk};
            fm = max4_abs(acc[j], fm);
        }
        return fm;
    }
    if (in_range) {
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            acc[j].x = divide_by_count(acc[j].x, fk, rk);
            acc[j].y = divide_by_count(acc[j].y, fk, rk);
            acc[j].z = divide_by_count(acc[j].z, fk, rk);
            acc[j].w = divide_by_count(acc[j].w, fk, rk);
            fm = max4_abs(acc[j], fm);
        }
        return fm;
    }
#pragma unroll
    for (int j = 0; j < Q; ++j) {
        acc[j].x = acc[j].x / fk;
        acc[j].y = acc[j].y / fk;
        acc[j].z = acc[j].z / fk;
        acc[j].w = acc[j].w / fk;
        fm = max4_abs(acc[j], fm);
    }
    return fm;
}

template <bool FASTDIV>
__device__ __forceinline__ uint32_t encode_one(const Search &sr, float x, float d, float r, bool recip)
{
    if (FASTDIV && recip) {
        uint32_t s0 = search_sum(sr, x * r);
        if (near_key(s0) > 2 * kNearWindow) return code_of(sr, s0, x);
    }
    return code_exact(sr, x, d);
}

// Copies the bucket table to LDS with all `n_threads` threads of the workgroup; the caller synchronises
// the workgroup before using it.
__device__ __forceinline__ Search load_bucket_table(const uint32_t *tab, uint32_t *lds, uint32_t n_threads = kWg)
{
    const uint32_t nbk = tab[kNBucketOff];
    for (uint32_t i = threadIdx.x; i < nbk; i += n_threads) lds[i] = tab[kBucketOff + i];
    return make_search(lds, tab[kLoKeyOff], nbk, tab[kHasMarksOff] != 0);
}

// Decode table in LDS, one copy per lane: entry (code, lane) at byte address code * 256 +
// lane * 4.  Lanes L and L + 32 share a bank but are served in different halves of the access,
// so a lookup never conflicts, and the address is two byte fields - code in byte 1, lane * 4 in
// byte 0 - which one v_perm_b32 assembles straight from a packed word of four codes.
// Thread t < 256 owns code t (workgroups have at least 256 threads).  The caller synchronises before the
// first lookup.
__device__ __forceinline__ void load_lut(const uint32_t *tab, float *lds)
{
    if (threadIdx.x < 256) {
        const float val = u2f(tab[kCbOff + threadIdx.x]);
        const v4f four = {val, val, val, val};
        v4f *row = reinterpret_cast<v4f *>(lds + threadIdx.x * kLutCopies);
#pragma unroll
        for (int c = 0; c < kLutCopies / 4; ++c) row[c] = four;
    }
}

// Table value of code number J (0..3) of the packed word w, for the lane whose byte offset
// into a table row is lane4 = lane * 4.
template <int J>
__device__ __forceinline__ float lut_at(const float *lut, uint32_t w, uint32_t lane4)
{
    const uint32_t addr = __builtin_amdgcn_perm(w, lane4, 0x0C0C0400u + (J << 8));
    return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lut) + addr);
}

__device__ __forceinline__ float lut_code(const float *lut, uint32_t code, uint32_t lane4)
{
    return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lut) + ((code << 8) | lane4));
}

// Element idx of an array whose base pointer is wave-uniform, addressed as "scalar base +
// 32-bit vector offset": the base is pinned to scalar registers, so that the compiler neither
// keeps a 64-bit address per lane nor hoists one out of the loop for every array it walks.
// The pointer goes through an integer on the way, which would make it a generic pointer; the
// cast names the global address space again (address space 1), so the access stays a global one.
#define DQ8_GLOBAL __attribute__((address_space(1)))

template <typename T>
__device__ __forceinline__ DQ8_GLOBAL T *uniform_global(T *p)
{
    const uintptr_t v = (uintptr_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (DQ8_GLOBAL T *)(((uintptr_t)hi << 32) | lo);
}

template <int NT, typename T>
__device__ __forceinline__ T ldg_at(const T *uniform_base, uint32_t idx)
{
    const DQ8_GLOBAL T *g = uniform_global(uniform_base);
    if constexpr (NT != 0)
        return __builtin_nontemporal_load(g + idx);
    else
        return g[idx];
}

// Store with the plain or non-temporal policy (the write-through policy of stg keeps its own form).
template <int NT, typename T>
__device__ __forceinline__ void stg_at(T *uniform_base, uint32_t idx, T v)
{
    DQ8_GLOBAL T *g = uniform_global(uniform_base);
    if constexpr (NT != 0)
        __builtin_nontemporal_store(v, g + idx);
    else
        g[idx] = v;
}

__device__ __forceinline__ uint32_t wave_in_wg() { return (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Index of this wavefront in the grid = the first unit it owns; held in scalar registers.
__device__ __forceinline__ size_t first_unit(int waves_per_wg = kWavesPerWg) { return (size_t)blockIdx.x * waves_per_wg + wave_in_wg(); }

// Maximum of |x[0..len)| over the elements this lane takes, for a unit that is short or not
// 16-byte aligned: whole quads with 128-bit loads when the start is aligned (the STRIDE lanes that
// share the unit take quads lane, lane + STRIDE, ...; a tail of fewer than four elements goes one by
// one), else element by element.
template <int NT, uint32_t STRIDE = kWave>
__device__ __forceinline__ uint32_t slow_absmax(const float *px, uint32_t len, uint32_t lane)
{
    uint32_t m = 0;
    uint32_t done = 0;
    if (((uintptr_t)px & 15) == 0) {
        const v4f *p4 = reinterpret_cast<const v4f *>(px);
        const uint32_t nq = len >> 2;
        float fm = 0.0f;
#pragma unroll 4
        for (uint32_t q = lane; q < nq; q += STRIDE) fm = max4_abs(ldg<NT>(p4 + q), fm);
        m = f2u(fm);
        done = nq << 2;
    }
    for (uint32_t i = done + lane; i < len; i += STRIDE) {
        const uint32_t a = abs_bits(px[i]);
        m = m > a ? m : a;
    }
    return m;
}

}  // namespace
