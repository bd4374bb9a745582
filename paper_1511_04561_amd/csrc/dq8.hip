// dq8 kernels and C ABI for gfx950 (MI355X).  See include/dq8.h for the contract.
//
// Work decomposition shared by every kernel: the array is cut into UNITS.  A unit is a run of
// at most U consecutive elements that lies inside one scale block, so one scale applies to the
// whole unit: unit u = (block b, chunk c) covers elements
// [b*B + c*U, min(b*B + (c+1)*U, (b+1)*B, n)).  A 64-lane wavefront (or, in the fused encoder,
// a team of four) owns a unit at a time and walks units with a grid-wide stride, so at any
// moment the whole chip streams through one narrow window of each array; the host sizes the
// grid so that every wavefront gets the same number of units and all of them are resident.
// U is 4096 where a whole block has to be held (fused encoder) and Q * 256 elsewhere, Q being
// the number of 128-bit accesses a lane keeps in flight.
//
// Inside a unit lane L owns elements 4*(64*it + L) .. +3: fp32 data moves as one 128-bit
// access per lane (1 KiB contiguous per wave instruction) and the matching four codes as one
// 32-bit access (256 B contiguous per instruction).  Units that are short, or whose addresses
// are not aligned for that, take a plain strided element loop with identical arithmetic.
// Every loop is software-pipelined: the loads of a wavefront's next unit are issued before
// the current one is processed.
//
// Built with -ffp-contract=off: the decode-and-average sum must round the product and the sum
// separately.  Divisions are the compiler's correctly rounded ones.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "dq8.h"
#include "dq8_internal.h"
#include "dq8_tables.hpp"

namespace {

using dq8::kBucketOff;
using dq8::kHasRemapOff;
using dq8::kRemapOff;
using dq8::kRemapWords;
using dq8::kCbOff;
using dq8::kLoKeyOff;
using dq8::kNBucketOff;
using dq8::kNearWindow;
using dq8::kTableWords;

constexpr int kWave = 64;
constexpr int kWavesPerWg = 4;
constexpr int kWg = kWave * kWavesPerWg;
constexpr int kUnit = 4096;                      // elements per unit
constexpr int kUnitQuads = kUnit / (4 * kWave);  // 16 quads per lane when one wave owns a unit
constexpr int kKinds = 4;
constexpr int kLutCopies = 64;                   // one copy of the decode table per lane
constexpr int kTeamSlots = 8;                    // LDS words for the cross-wave maximum (2 phases x 4 waves)

typedef float v4f __attribute__((ext_vector_type(4)));

// Tables of the three data types, one image per device (each GPU holds its own copy).
__device__ __align__(256) uint32_t g_tables[kKinds][kTableWords];

struct WorkerPtrs {
    const uint8_t *codes[DQ8_MAX_K];
    const float *scales[DQ8_MAX_K];
};

// ---------------------------------------------------------------- device helpers

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
__device__ __forceinline__ uint32_t cap_to_unit(size_t v)
{
    static_assert(U > 0 && (U & (U - 1)) == 0, "unit sizes are powers of two");
    return (v >> __builtin_ctz(U)) != 0 ? (uint32_t)U : (uint32_t)v;
}

template <int U>
__device__ __forceinline__ Unit unit_of(size_t u, size_t n, size_t B, size_t nb, size_t upb)
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

// Search state for the encoder (see dq8_tables.hpp): bucket table plus the clamp range, and
// for a data type with repeated values the table that turns a rank into its code.
struct Search {
    const uint32_t *bucket;  // LDS on the device
    const uint32_t *remap;   // NULL when every rank is its own code
    uint32_t lo_key;         // key of the first bucket
    float lo_f, hi_f;        // clamp range as binary32 values (bit patterns lo_bits, hi_bits)
};

__host__ __device__ __forceinline__ Search make_search(const uint32_t *bucket, uint32_t lo_key, uint32_t n_bucket,
                                                       const uint32_t *remap = nullptr)
{
    Search s;
    s.bucket = bucket;
    s.remap = remap;
    s.lo_key = lo_key;
    s.lo_f = u2f((lo_key << 16) + 0x8000u);
    s.hi_f = u2f(((lo_key + n_bucket - 1) << 16) + 0x8000u);
    return s;
}

// sum >> 16 = rank of the nearest table value (the number of thresholds <= |xn|), which is its
// magnitude field except for a type with a rank-to-code table (see finish_sum); the low half of
// sum measures the distance to the threshold of the bucket.  Non-negative binary32 values order like their bit patterns,
// so the clamp is done on the value.
__host__ __device__ __forceinline__ uint32_t search_sum(const Search &s, float xn)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const float c = __builtin_amdgcn_fmed3f(__builtin_fabsf(xn), s.lo_f, s.hi_f);
#else
    float c = __builtin_fabsf(xn);
    c = c >= s.lo_f ? c : s.lo_f;  // also takes NaN to the low end; inputs are finite anyway
    c = c <= s.hi_f ? c : s.hi_f;
#endif
    const uint32_t a = f2u(c);  // the low 16 bits of lo_base are zero: subtracting it only moves the key
    return s.bucket[(a >> 16) - s.lo_key] + (a & 0xFFFFu);
}

// Rank to magnitude field in bits 16..22, for the types where the two differ.  Kept out of
// search_sum so that an encoder takes this (wavefront-uniform) branch once per group of sums.
__host__ __device__ __forceinline__ uint32_t finish_sum(const Search &s, uint32_t sum) { return s.remap[sum >> 16] << 16; }

// (sum + W) mod 2^16 <= 2 W  <=>  |xn| is within W binary32 steps of a threshold or a bucket edge.
__host__ __device__ __forceinline__ uint32_t near_key(uint32_t sum) { return (sum + kNearWindow) & 0xFFFFu; }

// Code = magnitude index, bit 7 = sign bit of the input (the divisor is positive).
__host__ __device__ __forceinline__ uint32_t code_from(uint32_t sum, float x) { return (sum >> 16) | ((f2u(x) >> 24) & 0x80u); }

__host__ __device__ __forceinline__ uint32_t code_of(const Search &s, uint32_t sum, float x)
{
    if (s.remap) sum = finish_sum(s, sum);
    return code_from(sum, x);
}

__host__ __device__ __forceinline__ uint32_t code_exact(const Search &s, float x, float d) { return code_of(s, search_sum(s, x / d), x); }

// Four codes in one word: byte i = magnitude index of sum i (its byte 2) with the sign bit of
// x i (top bit of its byte 3).  v_perm_b32 gathers the bytes: selector byte 0..3 picks a byte
// of the second operand, 4..7 of the first, 0x0C gives zero.
__device__ __forceinline__ uint32_t pack_codes(const Search &sr, uint32_t s0, uint32_t s1, uint32_t s2, uint32_t s3, v4f v)
{
    if (sr.remap) {
        s0 = finish_sum(sr, s0);
        s1 = finish_sum(sr, s1);
        s2 = finish_sum(sr, s2);
        s3 = finish_sum(sr, s3);
    }
    const uint32_t m01 = __builtin_amdgcn_perm(s1, s0, 0x0C0C0602u);
    const uint32_t m23 = __builtin_amdgcn_perm(s3, s2, 0x06020C0Cu);
    const uint32_t g01 = __builtin_amdgcn_perm(f2u(v.y), f2u(v.x), 0x0C0C0703u);
    const uint32_t g23 = __builtin_amdgcn_perm(f2u(v.w), f2u(v.z), 0x07030C0Cu);
    return ((g01 | g23) & 0x80808080u) | m01 | m23;
}

// A scale qualifies for the reciprocal path when 1/d and every product x * (1/d) that can
// reach a threshold are normal numbers: 2^-100 <= d <= 2^100.
__host__ __device__ __forceinline__ bool reciprocal_ok(float d)
{
    uint32_t b = f2u(d);
    return b >= 0x0D800000u && b <= 0x71800000u;
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
    return pack_codes(sr, search_sum(sr, v.x / d), search_sum(sr, v.y / d), search_sum(sr, v.z / d), search_sum(sr, v.w / d), v);
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

// Copies the bucket table (and the rank-to-code table of a type that has one, right behind it)
// to LDS with all `n_threads` threads of the workgroup; the caller synchronises the workgroup
// before using it.
__device__ __forceinline__ Search load_bucket_table(const uint32_t *tab, uint32_t *lds, uint32_t n_threads = kWg)
{
    const uint32_t nbk = tab[kNBucketOff];
    for (uint32_t i = threadIdx.x; i < nbk; i += n_threads) lds[i] = tab[kBucketOff + i];
    const uint32_t *remap = nullptr;
    if (tab[kHasRemapOff]) {
        for (uint32_t i = threadIdx.x; i < (uint32_t)kRemapWords; i += n_threads) lds[nbk + i] = tab[kRemapOff + i];
        remap = lds + nbk;
    }
    return make_search(lds, tab[kLoKeyOff], nbk, remap);
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

// ---------------------------------------------------------------- kernels

__global__ void k_fill_zero(float *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// Plain fp32 copy with the access pattern of the codec kernels (units of Q * 256 elements,
// 128-bit accesses).  Exists to calibrate bandwidth and hardware-counter readings against a
// kernel whose traffic is known exactly: 4 bytes read and 4 bytes written per element.
template <int Q, int NT>
__global__ __launch_bounds__(kWg) void k_copy(const float *__restrict__ src, float *__restrict__ dst, size_t n,
                                             size_t n_units, size_t n_waves)
{
    constexpr int U = Q * 4 * kWave;
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of<U>(u, n, n, 1, 0);
        const float *ps = src + un.start;
        float *pd = dst + un.start;
        if (un.len == U && (((uintptr_t)ps | (uintptr_t)pd) & 15) == 0) {
            const v4f *s4 = reinterpret_cast<const v4f *>(ps);
            v4f *d4 = reinterpret_cast<v4f *>(pd);
            v4f v[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) v[j] = ldg<NT>(s4 + j * kWave + lane);
#pragma unroll
            for (int j = 0; j < Q; ++j) stg<NT>(d4 + j * kWave + lane, v[j]);
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) pd[i] = ps[i];
        }
    }
}

// Block maxima.  One wavefront per unit of Q * 256 elements.  upb == 1: each unit is a whole
// block and stores its maximum.  upb > 1: scales[] was zeroed and the pieces of a block merge
// with an integer atomic max (non-negative binary32 numbers order like their bit patterns).
// per_wave == 0: wavefront w takes units w, w + n_waves, ...  per_wave > 0 (used when blocks span
// several units): it takes the per_wave consecutive units from w * per_wave on, keeps one
// running maximum per lane while the block stays the same and issues one atomic per block it
// touches -- thousands of atomics on one address cost more than reading the array.
template <int Q, int NT>
__global__ __launch_bounds__(kWg) void k_absmax(const float *__restrict__ x, size_t n, size_t B, size_t nb, size_t upb,
                                               size_t n_units, size_t n_waves, size_t per_wave, float *__restrict__ scales)
{
    constexpr int U = Q * 4 * kWave;
    const uint32_t lane = threadIdx.x & 63;
    const size_t w = first_unit();
    size_t u = per_wave ? w * per_wave : w;
    const size_t stride = per_wave ? 1 : n_waves;
    const size_t end = per_wave ? (u + per_wave < n_units ? u + per_wave : n_units) : n_units;
    Unit un;
    bool fast = false;
    v4f v[Q];
    auto open_unit = [&](size_t uu, Unit &q, bool &f) {
        q = unit_of<U>(uu, n, B, nb, upb);
        f = q.len == U && ((uintptr_t)(x + q.start) & 15) == 0;
        if (f) {
            const v4f *p4 = reinterpret_cast<const v4f *>(x + q.start);
#pragma unroll
            for (int j = 0; j < Q; ++j) v[j] = ldg<NT>(p4 + j * kWave + lane);
        }
    };
    if (u < end) open_unit(u, un, fast);
    uint32_t run = 0;  // this lane's maximum over the units of the current block so far
    while (u < end) {
        uint32_t m;
        if (fast) {
            float fm = 0.0f;
#pragma unroll
            for (int j = 0; j < Q; ++j) fm = max4_abs(v[j], fm);
            m = f2u(fm);
        } else {
            m = slow_absmax<NT>(x + un.start, un.len, lane);
        }
        const size_t blk = un.block;
        u += stride;
        const bool more = u < end;
        if (more) open_unit(u, un, fast);  // next unit's loads fly during the reduction
        run = run > m ? run : m;
        if (!more || un.block != blk) {
            const uint32_t r = wave_max_u32(run);
            run = 0;
            if (lane == 0) {
                if (upb == 1)
                    scales[blk] = u2f(r);
                else
                    atomicMax(reinterpret_cast<unsigned int *>(scales) + blk, r);
            }
        }
    }
}

// Compression.  A team of WPB wavefronts owns a unit of WPB * QL * 256 elements, QL quads per lane:
// WPB == 1, each wavefront of the workgroup walks its own units; WPB == 4, the workgroup's four
// wavefronts share a unit and combine their maxima through LDS.
// FUSED: a unit is a whole block (upb == 1); the team reduces the block's maximum from
// registers, stores it and quantises the same registers.  Otherwise the scale of the unit's
// block is read from scales[].
// The loop is software-pipelined: the loads of a team's next unit are issued before the
// current unit is reduced and quantised, so each wavefront always has loads in flight.
// A unit shorter than that (a block that is not a power of two, the end of a block or of the
// array) takes the same path when it consists of whole aligned quads: a lane whose quad lies
// past the end loads the unit's last quad instead (an unconditional load of valid memory: the
// maximum does not change and the lane stores nothing).
template <int WPB, int QL, int NT, bool FUSED, bool FASTDIV>
struct Encoder {
    static constexpr int Q = QL;
    static constexpr uint32_t TEAM = kWave * WPB;
    static constexpr int U = QL * 4 * (int)TEAM;

    const float *x;
    uint8_t *codes;
    float *scales;
    size_t n, B, nb, upb;
    uint32_t *slots;
    Search sr;
    uint32_t lane, wave, tl, phase;

    struct Slot {
        Unit un;
        bool fast;
        v4f v[Q];
    };

    __device__ __forceinline__ void fetch(size_t u, Slot &sl) const
    {
        sl.un = unit_of<U>(u, n, B, nb, upb);
        const float *px = x + sl.un.start;
        sl.fast = sl.un.len >= 4 && (sl.un.len & 3) == 0 && ((uintptr_t)px & 15) == 0 &&
                  ((uintptr_t)(codes + sl.un.start) & 3) == 0;
        if (sl.fast) {
            const v4f *p4 = reinterpret_cast<const v4f *>(px);
            const uint32_t last = (sl.un.len >> 2) - 1;
#pragma unroll
            for (int it = 0; it < Q; ++it) {
                const uint32_t q = it * TEAM + tl;
                sl.v[it] = ldg<NT>(p4 + (q < last ? q : last));
            }
        }
    }

    __device__ __forceinline__ void process(Slot &sl)
    {
        const Unit &un = sl.un;
        const float *px = x + un.start;
        uint8_t *pc = codes + un.start;
        float s;
        if (FUSED) {
            uint32_t m;
            if (sl.fast) {
                float fm = 0.0f;
#pragma unroll
                for (int it = 0; it < Q; ++it) fm = max4_abs(sl.v[it], fm);
                m = f2u(fm);
            } else {
                m = slow_absmax<NT, TEAM>(px, un.len, tl);
            }
            m = wave_max_u32(m);
            if (WPB > 1) {
                if (lane == 0) slots[phase * kWavesPerWg + wave] = m;
                __syncthreads();  // every wavefront of the workgroup walks the same units
                const uint32_t *sp = slots + phase * kWavesPerWg;
                uint32_t a = sp[0] > sp[1] ? sp[0] : sp[1], b = sp[2] > sp[3] ? sp[2] : sp[3];
                m = (uint32_t)__builtin_amdgcn_readfirstlane((int)(a > b ? a : b));
                phase ^= 1;  // the other half of slots next time: one barrier per unit is enough
            }
            s = u2f(m);
            if (tl == 0) scales[un.block] = s;
        } else {
            s = scales[un.block];
        }
        const float d = s == 0.0f ? 1.0f : s;  // a zero scale leaves the value as it is
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        if (sl.fast) {
            uint32_t *c4 = reinterpret_cast<uint32_t *>(pc);
            const uint32_t nq = un.len >> 2;
#pragma unroll
            for (int it = 0; it < Q; ++it) {
                const uint32_t cw = encode_quad<FASTDIV>(sr, sl.v[it], d, r, recip);
                if (it * TEAM + tl < nq) stg<NT>(c4 + it * TEAM + tl, cw);
            }
        } else {
            // a misaligned unit or one that does not consist of whole quads: whole quads where the addresses allow (the lanes of the team take quads
            // tl, tl + TEAM, ...), the rest element by element
            uint32_t done = 0;
            if ((((uintptr_t)px & 15) | ((uintptr_t)pc & 3)) == 0) {
                const v4f *p4 = reinterpret_cast<const v4f *>(px);
                uint32_t *c4 = reinterpret_cast<uint32_t *>(pc);
                const uint32_t nq = un.len >> 2;
                for (uint32_t q = tl; q < nq; q += TEAM) stg<NT>(c4 + q, encode_quad<FASTDIV>(sr, ldg<NT>(p4 + q), d, r, recip));
                done = nq << 2;
            }
            for (uint32_t i = done + tl; i < un.len; i += TEAM) pc[i] = (uint8_t)encode_one<FASTDIV>(sr, px[i], d, r, recip);
        }
    }
};

template <int WPB, int QL, int NT, bool FUSED, bool FASTDIV>
__global__ __launch_bounds__(kWg) void k_encode(const uint32_t *__restrict__ tab, const float *__restrict__ x, size_t n,
                                               size_t B, size_t nb, size_t upb, size_t n_units, size_t n_teams,
                                               float *__restrict__ scales, uint8_t *__restrict__ codes)
{
    static_assert(WPB == 1 || WPB == kWavesPerWg, "a team is one wavefront or the whole workgroup");
    using Enc = Encoder<WPB, QL, NT, FUSED, FASTDIV>;
    extern __shared__ uint32_t lds[];
    Enc e;
    e.x = x;
    e.codes = codes;
    e.scales = scales;
    e.n = n;
    e.B = B;
    e.nb = nb;
    e.upb = upb;
    e.slots = lds;  // kTeamSlots words, then the bucket table
    e.lane = threadIdx.x & 63;
    e.wave = wave_in_wg();
    e.tl = WPB == 1 ? e.lane : threadIdx.x;
    e.phase = 0;
    size_t u = WPB == 1 ? first_unit() : (size_t)blockIdx.x;
    typename Enc::Slot a, b;
    if (u < n_units) e.fetch(u, a);  // the first loads are in flight while the table is copied
    e.sr = load_bucket_table(tab, lds + kTeamSlots);
    __syncthreads();
    while (u < n_units) {
        size_t nx = u + n_teams;
        if (nx < n_units) e.fetch(nx, b);
        e.process(a);
        u = nx;
        if (!(u < n_units)) break;
        nx = u + n_teams;
        if (nx < n_units) e.fetch(nx, a);
        e.process(b);
        u = nx;
    }
}

// Compression of whole, aligned blocks of 4096 elements: the common case of k_encode<4, NT, true,
// FASTDIV> (a team of four wavefronts per block, maximum and quantisation from registers) with
// nothing else in the loop.  Block b starts at element 4096 b, x is 16-byte and codes 4-byte
// aligned, so unit geometry is a multiplication and there is no slow path to branch around.
// A ragged last block of tail_len elements is done by the last workgroup after its loop.
// REMAP = false promises a type without a rank-to-code table: the test for one drops out of the loop.
template <int NT, bool FASTDIV, bool REMAP>
__global__ __launch_bounds__(kWg) void k_encode_full(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                    uint32_t n_full, uint32_t n_teams, uint32_t tail_len,
                                                    float *__restrict__ scales, uint8_t *__restrict__ codes)
{
    constexpr int Q = kUnitQuads / kWavesPerWg;
    extern __shared__ uint32_t lds[];
    uint32_t *slots = lds;  // kTeamSlots words, then the bucket table
    const uint32_t lane = threadIdx.x & 63, wave = wave_in_wg(), tl = threadIdx.x;
    uint32_t phase = 0;
    Search sr;
    auto fetch = [&](uint32_t u, v4f(&v)[Q]) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x) + (size_t)u * (kUnit / 4);
#pragma unroll
        for (int it = 0; it < Q; ++it) v[it] = ldg_at<NT>(p4, it * kWg + tl);
    };
    // Maximum over the team of the wave maxima m, through LDS; one barrier per call.
    auto team_max = [&](uint32_t m) {
        if (lane == 0) slots[phase * kWavesPerWg + wave] = m;
        __syncthreads();
        const uint32_t *sp = slots + phase * kWavesPerWg;
        const uint32_t a = sp[0] > sp[1] ? sp[0] : sp[1], b = sp[2] > sp[3] ? sp[2] : sp[3];
        phase ^= 1;  // the other half of slots next time
        return (uint32_t)__builtin_amdgcn_readfirstlane((int)(a > b ? a : b));
    };
    auto process = [&](uint32_t u, v4f(&v)[Q]) {
        float fm = 0.0f;
#pragma unroll
        for (int it = 0; it < Q; ++it) fm = max4_abs(v[it], fm);
        const float s = u2f(team_max(wave_max_u32(f2u(fm))));
        if (tl == 0) scales[u] = s;
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes) + (size_t)u * (kUnit / 4);
#pragma unroll
        for (int it = 0; it < Q; ++it) stg_at<NT>(c4, it * kWg + tl, encode_quad<FASTDIV>(sr, v[it], d, r, recip));
    };
    uint32_t u = blockIdx.x;
    v4f a[Q], b[Q];
    if (u < n_full) fetch(u, a);  // the first loads are in flight while the table is copied
    sr = load_bucket_table(tab, lds + kTeamSlots);
    if (!REMAP) sr.remap = nullptr;
    __syncthreads();
    // Steady state: the fetch of the next block is unconditional and comes before the work on the
    // current one, so at the point where the current block's registers are first read the compiler
    // knows exactly how many younger loads are outstanding and waits for the older ones only.  (A
    // fetch under "if there is a next block" merges with the path that has none, and the merged
    // state makes it wait for the loads it has just issued.)  The last block of a team is done
    // outside the steady state.
    if (u < n_full) {
        for (;;) {
            uint32_t nx = u + n_teams;
            if (!(nx < n_full)) {
                process(u, a);
                break;
            }
            fetch(nx, b);
            process(u, a);
            u = nx;
            nx = u + n_teams;
            if (!(nx < n_full)) {
                process(u, b);
                break;
            }
            fetch(nx, a);
            process(u, b);
            u = nx;
        }
    }
    if (tail_len != 0 && blockIdx.x == gridDim.x - 1) {
        const float *px = x + (size_t)n_full * kUnit;
        uint8_t *pc = codes + (size_t)n_full * kUnit;
        uint32_t m = 0;
        for (uint32_t i = tl; i < tail_len; i += kWg) {
            const uint32_t v = abs_bits(px[i]);
            m = m > v ? m : v;
        }
        const float s = u2f(team_max(wave_max_u32(m)));
        if (tl == 0) scales[n_full] = s;
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        for (uint32_t i = tl; i < tail_len; i += kWg) pc[i] = (uint8_t)encode_one<FASTDIV>(sr, px[i], d, r, recip);
    }
}

// Decompression of one buffer: out = table[code] * scale.  One wavefront per unit of Q * 256
// elements: Q code words (4 codes each) per lane; the next unit's words are loaded before the
// current ones are expanded.
// RAGGED = true (chosen by the host when blocks are not whole units): a unit of fewer whole aligned
// quads stays on this path; a lane whose quad lies past the end loads the unit's last code word
// instead (unconditional, valid memory) and stores nothing.
template <int Q, int NT, int WPW, bool RAGGED>
__global__ __launch_bounds__(kWave * WPW) void k_decode(const uint32_t *__restrict__ tab, const uint8_t *__restrict__ codes,
                                                       const float *__restrict__ scales, size_t n, size_t B, size_t nb,
                                                       size_t upb, size_t n_units, size_t n_waves, float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    size_t u = first_unit(WPW);
    Unit un;
    bool fast = false;
    uint32_t w[Q];
    auto open_unit = [&](size_t uu, Unit &q, bool &f) {
        q = unit_of<U>(uu, n, B, nb, upb);
        f = ((uintptr_t)(out + q.start) & 15) == 0 && ((uintptr_t)(codes + q.start) & 3) == 0;
        f = f && (RAGGED ? (q.len >= 4 && (q.len & 3) == 0) : q.len == U);
        if (f) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(codes + q.start);
            const uint32_t last = (q.len >> 2) - 1;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const uint32_t i = j * kWave + lane;
                w[j] = ldg<NT>(c4 + (RAGGED ? (i < last ? i : last) : i));
            }
        }
    };
    if (u < n_units) open_unit(u, un, fast);  // the first loads are in flight while the table is built
    load_lut(tab, lut);
    __syncthreads();
    while (u < n_units) {
        const float s = scales[un.block];
        float *po = out + un.start;
        if (fast) {
            uint32_t cur[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) cur[j] = w[j];
            const uint32_t nq = un.len >> 2;
            u += n_waves;
            if (u < n_units) open_unit(u, un, fast);
            v4f *o4 = reinterpret_cast<v4f *>(po);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                v4f r;
                r.x = lut_at<0>(lut, cur[j], lane4) * s;
                r.y = lut_at<1>(lut, cur[j], lane4) * s;
                r.z = lut_at<2>(lut, cur[j], lane4) * s;
                r.w = lut_at<3>(lut, cur[j], lane4) * s;
                if (!RAGGED || j * kWave + lane < nq) stg<NT>(o4 + j * kWave + lane, r);
            }
        } else {
            // a short or misaligned unit: whole quads with 128-bit stores where the addresses allow, the rest
            // element by element
            const uint8_t *pc = codes + un.start;
            uint32_t done = 0;
            if ((((uintptr_t)po & 15) | ((uintptr_t)pc & 3)) == 0) {
                const uint32_t *c4 = reinterpret_cast<const uint32_t *>(pc);
                v4f *o4 = reinterpret_cast<v4f *>(po);
                const uint32_t nq = un.len >> 2;
                for (uint32_t q = lane; q < nq; q += kWave) {
                    const uint32_t cw = ldg<NT>(c4 + q);
                    v4f r;
                    r.x = lut_at<0>(lut, cw, lane4) * s;
                    r.y = lut_at<1>(lut, cw, lane4) * s;
                    r.z = lut_at<2>(lut, cw, lane4) * s;
                    r.w = lut_at<3>(lut, cw, lane4) * s;
                    stg<NT>(o4 + q, r);
                }
                done = nq << 2;
            }
            for (uint32_t i = done + lane; i < un.len; i += kWave) po[i] = lut_code(lut, pc[i], lane4) * s;
            u += n_waves;
            if (u < n_units) open_unit(u, un, fast);
        }
    }
}

// Decompress K buffers and average: acc = +0; acc += table[code_k] * scale_k for k = 0..K-1
// in order; out = acc / K.  KT > 0 fixes K at compile time (fully unrolled, Q code words per
// lane and worker per unit, next unit's words requested before the current ones are used);
// KT == 0 reads K from the argument.
template <int KT, int Q, int NT, int WPW>
__global__ __launch_bounds__(kWave * WPW) void k_decode_avg(const uint32_t *__restrict__ tab, WorkerPtrs p, int K_rt,
                                                           size_t n, size_t B, size_t nb, size_t upb, size_t n_units,
                                                           size_t n_waves, float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int KA = KT > 0 ? KT : 1;
    constexpr int U = Q * 4 * kWave;
    const int K = KT > 0 ? KT : K_rt;
    const float fk = (float)K;
    // For K a power of two, 1/K is exact and acc * (1/K) is the correctly rounded value of the
    // same real number as acc / K (subnormal results and signed zeros included), at the cost
    // of one multiplication instead of a division sequence.
    const bool pow2 = (K & (K - 1)) == 0;
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    size_t u = first_unit(WPW);
    Unit un;
    bool fast = false;     // whole quads at aligned addresses
    bool aligned = false;  // 128-bit stores and 32-bit code loads are possible
    uint32_t w[KA][Q];
    auto open_unit = [&](size_t uu, Unit &q, bool &f, bool &al) {
        q = unit_of<U>(uu, n, B, nb, upb);
        al = ((uintptr_t)(out + q.start) & 15) == 0;
        for (int k = 0; k < K; ++k) al = al && (((uintptr_t)(p.codes[k] + q.start) & 3) == 0);
        // a unit of fewer whole quads stays on the pipelined path: a lane whose quad lies past the end loads
        // the unit's last code word instead (unconditional, valid memory) and stores nothing
        f = al && q.len >= 4 && (q.len & 3) == 0;
        if (KT > 0 && f) {
            const uint32_t last = (q.len >> 2) - 1;
#pragma unroll
            for (int k = 0; k < KA; ++k) {
                const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k] + q.start);
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const uint32_t i = j * kWave + lane;
                    w[k][j] = ldg<NT>(c4 + (i < last ? i : last));
                }
            }
        }
    };
    if (u < n_units) open_unit(u, un, fast, aligned);
    load_lut(tab, lut);
    __syncthreads();
    while (u < n_units) {
        float *po = out + un.start;
        if (fast && KT > 0) {
            float sc[KA];
#pragma unroll
            for (int k = 0; k < KA; ++k) sc[k] = p.scales[k][un.block];
            uint32_t cur[KA][Q];
#pragma unroll
            for (int k = 0; k < KA; ++k)
#pragma unroll
                for (int j = 0; j < Q; ++j) cur[k][j] = w[k][j];
            const uint32_t nq = un.len >> 2;
            u += n_waves;
            if (u < n_units) open_unit(u, un, fast, aligned);
            v4f *o4 = reinterpret_cast<v4f *>(po);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int k = 0; k < KA; ++k) {
                    a.x = a.x + lut_at<0>(lut, cur[k][j], lane4) * sc[k];
                    a.y = a.y + lut_at<1>(lut, cur[k][j], lane4) * sc[k];
                    a.z = a.z + lut_at<2>(lut, cur[k][j], lane4) * sc[k];
                    a.w = a.w + lut_at<3>(lut, cur[k][j], lane4) * sc[k];
                }
                a.x = mean_of(a.x);
                a.y = mean_of(a.y);
                a.z = mean_of(a.z);
                a.w = mean_of(a.w);
                if (j * kWave + lane < nq) stg<NT>(o4 + j * kWave + lane, a);
            }
        } else {
            // any K, and misaligned units or units that are not whole quads: whole quads where the addresses allow (lanes take quads
            // lane, lane + 64, ...), the rest element by element
            uint32_t done = 0;
            if (aligned) {
                v4f *o4 = reinterpret_cast<v4f *>(po);
                const uint32_t nq = un.len >> 2;
                for (uint32_t q = lane; q < nq; q += kWave) {
                    v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
                    for (int k = 0; k < K; ++k) {
                        const uint32_t ww = ldg<NT>(reinterpret_cast<const uint32_t *>(p.codes[k] + un.start) + q);
                        const float s = p.scales[k][un.block];
                        a.x = a.x + lut_at<0>(lut, ww, lane4) * s;
                        a.y = a.y + lut_at<1>(lut, ww, lane4) * s;
                        a.z = a.z + lut_at<2>(lut, ww, lane4) * s;
                        a.w = a.w + lut_at<3>(lut, ww, lane4) * s;
                    }
                    a.x = mean_of(a.x);
                    a.y = mean_of(a.y);
                    a.z = mean_of(a.z);
                    a.w = mean_of(a.w);
                    stg<NT>(o4 + q, a);
                }
                done = nq << 2;
            }
            for (uint32_t i = done + lane; i < un.len; i += kWave) {
                float a = 0.0f;
                for (int k = 0; k < K; ++k) a = a + lut_code(lut, p.codes[k][un.start + i], lane4) * p.scales[k][un.block];
                po[i] = mean_of(a);
            }
            u += n_waves;
            if (u < n_units) open_unit(u, un, fast, aligned);
        }
    }
}

// K-way decode-and-average of whole, aligned units, K = 2, 4 or 8: the common case of
// k_decode_avg with nothing else in the loop.  Unit u covers elements [U u, U (u + 1)), U divides
// the block size and block / U is a power of two, so a unit's block is u >> block_shift; out is
// 16-byte and every code buffer 4-byte aligned.  The K scales of a unit travel with its code
// words (read at the start of the unit's work they would cost a memory round trip per unit),
// and the fetch of the next unit is unconditional in the steady state, so the compiler waits
// for exactly the loads it needs.  A ragged last unit of tail_len elements is done by one
// wavefront of the last workgroup after its loop.
// LOCAL: an fp32 array (16-byte aligned) is the first term of every sum and the divisor is K + 1.
template <int KT, int Q, int NT, int WPW, bool LOCAL>
__global__ __launch_bounds__(kWave * WPW) void k_decode_avg_full(const uint32_t *__restrict__ tab, WorkerPtrs p,
                                                                const float *__restrict__ local, uint32_t n_full,
                                                                uint32_t n_waves, uint32_t block_shift, uint32_t tail_len,
                                                                float *__restrict__ out)
{
    static_assert(KT == 2 || KT == 4 || KT == 8, "unrolled for these K");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    constexpr float fk = (float)(KT + (LOCAL ? 1 : 0));
    constexpr float rk = 1.0f / (float)KT;  // acc * (1 / K) equals acc / K exactly for a power of two
    auto mean_of = [&](float acc) { return LOCAL ? acc / fk : acc * rk; };
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    struct Slot {
        uint32_t w[KT][Q];
        float sw[KT];
        v4f loc[LOCAL ? Q : 1];
    };
    auto fetch = [&](uint32_t u, Slot &sl) {
        if (LOCAL) {
            const v4f *l4 = reinterpret_cast<const v4f *>(local) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) sl.loc[j] = ldg_at<NT>(l4, j * kWave + lane);
        }
#pragma unroll
        for (int k = 0; k < KT; ++k) sl.sw[k] = p.scales[k][u >> block_shift];
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k]) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) sl.w[k][j] = ldg_at<NT>(c4, j * kWave + lane);
        }
    };
    auto process = [&](uint32_t u, Slot &sl) {
        float sc[KT];
#pragma unroll
        for (int k = 0; k < KT; ++k) sc[k] = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(sl.sw[k])));
        v4f *o4 = reinterpret_cast<v4f *>(out) + (size_t)u * (U / 4);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
            if (LOCAL) {  // the sum starts at +0: a local -0 becomes +0
                a.x = a.x + sl.loc[j].x;
                a.y = a.y + sl.loc[j].y;
                a.z = a.z + sl.loc[j].z;
                a.w = a.w + sl.loc[j].w;
            }
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                a.x = a.x + lut_at<0>(lut, sl.w[k][j], lane4) * sc[k];
                a.y = a.y + lut_at<1>(lut, sl.w[k][j], lane4) * sc[k];
                a.z = a.z + lut_at<2>(lut, sl.w[k][j], lane4) * sc[k];
                a.w = a.w + lut_at<3>(lut, sl.w[k][j], lane4) * sc[k];
            }
            a.x = mean_of(a.x);
            a.y = mean_of(a.y);
            a.z = mean_of(a.z);
            a.w = mean_of(a.w);
            stg<NT>(o4 + j * kWave + lane, a);
        }
    };
    uint32_t u = (uint32_t)first_unit(WPW);
    Slot a, b;
    if (u < n_full) fetch(u, a);  // the first loads are in flight while the table is built
    load_lut(tab, lut);
    __syncthreads();
    if (u < n_full) {
        for (;;) {
            uint32_t nx = u + n_waves;
            if (!(nx < n_full)) {
                process(u, a);
                break;
            }
            fetch(nx, b);
            process(u, a);
            u = nx;
            nx = u + n_waves;
            if (!(nx < n_full)) {
                process(u, b);
                break;
            }
            fetch(nx, a);
            process(u, b);
            u = nx;
        }
    }
    if (tail_len != 0 && blockIdx.x == gridDim.x - 1 && wave_in_wg() == 0) {
        const size_t start = (size_t)n_full * U;
        const size_t blk = n_full >> block_shift;
        for (uint32_t i = lane; i < tail_len; i += kWave) {
            float acc = 0.0f;
            if (LOCAL) acc = acc + local[start + i];
#pragma unroll
            for (int k = 0; k < KT; ++k) acc = acc + lut_code(lut, p.codes[k][start + i], lane4) * p.scales[k][blk];
            out[start + i] = mean_of(acc);
        }
    }
}

// Average of K workers' buffers (plus, optionally, a local fp32 array as the first term) with a
// whole unit of 4096 elements held in one wavefront's registers: 16 quads of running sums per
// lane, the workers added one after the other while the next worker's code words are in flight.
// The means can be stored as fp32 (mean_out) and / or compressed again from the registers
// (codes_out, scales_out; needs a unit to be a whole scale block, upb == 1): the second round of
// the gradient exchange then reads K bytes and writes one byte per element instead of going
// through an fp32 array in memory.  Arithmetic and order are those of k_decode_avg followed by
// k_encode, so the results are identical to the two calls.
// Two workgroups of WPW wavefronts share a compute unit (each holds the 64 KiB decode table),
// so the register budget per lane is 512 / (WPW / 2): 170 for six wavefronts, 128 for eight.
// The unit is QL * 256 elements (the host picks the smallest that holds a block, up to 4096).
// RAGGED = true (chosen by the host when blocks are not whole units): a unit of fewer whole aligned
// quads stays on the register path; a lane whose quad lies past the end loads the unit's last quad
// instead (unconditional loads of valid memory; the maximum does not change) and stores nothing.
// This costs a register per quad for the clamped offsets, which the kernel for whole units cannot spare.
template <int QL, int NT, bool FASTDIV, int WPW, bool RAGGED>
__global__ __launch_bounds__(kWave * WPW, WPW / 2) void k_avg_block(const uint32_t *__restrict__ tab, WorkerPtrs p, int K,
                                                          const float *__restrict__ local, size_t n, size_t B,
                                                          size_t nb, size_t upb, size_t n_units, size_t n_waves,
                                                          float *__restrict__ mean_out, float *__restrict__ scales_out,
                                                          uint8_t *__restrict__ codes_out)
{
    static_assert(WPW >= 4, "the decode table is filled by 256 threads");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t bucket_lds[];
    constexpr int Q = QL;
    constexpr int U = QL * 4 * kWave;
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    load_lut(tab, lut);
    Search sr = make_search(bucket_lds, tab[kLoKeyOff], tab[kNBucketOff]);
    if (codes_out) sr = load_bucket_table(tab, bucket_lds, kWave * WPW);
    __syncthreads();
    for (size_t u = first_unit(WPW); u < n_units; u += n_waves) {
        const Unit un = unit_of<U>(u, n, B, nb, upb);
        bool aligned = true;  // 128-bit accesses to the fp32 arrays and 32-bit ones to the codes are possible
        for (int k = 0; k < K; ++k) aligned = aligned && (((uintptr_t)(p.codes[k] + un.start) & 3) == 0);
        if (local) aligned = aligned && (((uintptr_t)(local + un.start) & 15) == 0);
        if (mean_out) aligned = aligned && (((uintptr_t)(mean_out + un.start) & 15) == 0);
        if (codes_out) aligned = aligned && (((uintptr_t)(codes_out + un.start) & 3) == 0);
        const bool fast = aligned && (RAGGED ? (un.len >= 4 && (un.len & 3) == 0) : un.len == (uint32_t)U);
        if (fast) {
            const uint32_t nq = un.len >> 2, last = nq - 1;
            auto qi = [&](int j) {  // this lane's j-th quad, clamped to the unit
                const uint32_t i = j * kWave + lane;
                return RAGGED ? (i < last ? i : last) : i;
            };
            v4f acc[Q];
            uint32_t wa[Q], wb[Q];
            auto load_w = [&](uint32_t(&w)[Q], int k) {
                const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k] + un.start);
#pragma unroll
                for (int j = 0; j < Q; ++j) w[j] = ldg_at<NT>(c4, qi(j));  // scalar base + 32-bit offset
            };
            auto add_w = [&](const uint32_t(&w)[Q], int k) {
                const float s = p.scales[k][un.block];
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    acc[j].x = acc[j].x + lut_at<0>(lut, w[j], lane4) * s;
                    acc[j].y = acc[j].y + lut_at<1>(lut, w[j], lane4) * s;
                    acc[j].z = acc[j].z + lut_at<2>(lut, w[j], lane4) * s;
                    acc[j].w = acc[j].w + lut_at<3>(lut, w[j], lane4) * s;
                }
                // pin the sums here, or the compiler defers them and holds the products of several workers
#pragma unroll
                for (int j = 0; j < Q; ++j) asm volatile("" : "+v"(acc[j].x), "+v"(acc[j].y), "+v"(acc[j].z), "+v"(acc[j].w));
            };
            if (K > 0) load_w(wa, 0);
            if (local) {
                const v4f *l4 = reinterpret_cast<const v4f *>(local + un.start);
#pragma unroll
                for (int j = 0; j < Q; ++j) acc[j] = ldg_at<NT>(l4, qi(j));
#pragma unroll
                for (int j = 0; j < Q; ++j) {  // the sum starts at +0: a local -0 becomes +0
                    acc[j].x = 0.0f + acc[j].x;
                    acc[j].y = 0.0f + acc[j].y;
                    acc[j].z = 0.0f + acc[j].z;
                    acc[j].w = 0.0f + acc[j].w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < Q; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
            }
            for (int k = 0; k < K; k += 2) {
                const bool more = k + 1 < K;
                if (more) load_w(wb, k + 1);
                add_w(wa, k);
                if (more) {
                    if (k + 2 < K) load_w(wa, k + 2);
                    add_w(wb, k + 1);
                }
            }
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                acc[j].x = mean_of(acc[j].x);
                acc[j].y = mean_of(acc[j].y);
                acc[j].z = mean_of(acc[j].z);
                acc[j].w = mean_of(acc[j].w);
            }
            if (mean_out) {
                v4f *o4 = reinterpret_cast<v4f *>(mean_out + un.start);
#pragma unroll
                for (int j = 0; j < Q; ++j)
                    if (!RAGGED || j * kWave + lane < nq) stg<NT>(o4 + j * kWave + lane, acc[j]);
            }
            if (codes_out) {
                float fm = 0.0f;
#pragma unroll
                for (int j = 0; j < Q; ++j) fm = max4_abs(acc[j], fm);
                const float s = u2f(wave_max_u32(f2u(fm)));
                if (lane == 0) scales_out[un.block] = s;
                const float d = s == 0.0f ? 1.0f : s;
                const float r = 1.0f / d;
                const bool recip = reciprocal_ok(d);
                uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out + un.start);
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const uint32_t cw = encode_quad<FASTDIV>(sr, acc[j], d, r, recip);
                    if (!RAGGED || j * kWave + lane < nq) stg<1>(c4 + j * kWave + lane, cw);
                }
            }
        } else {
            // A misaligned unit or one that is not whole quads.  Whole quads where the addresses allow (lanes take quads lane,
            // lane + 64, ...), the remaining elements one by one.  The means are formed again for each use
            // (store, maximum, compression) rather than kept.
            const uint32_t nq = aligned ? un.len >> 2 : 0;
            const uint32_t done = nq << 2;
            auto mean_at = [&](uint32_t i) {
                float a = 0.0f;
                if (local) a = a + local[un.start + i];
                for (int k = 0; k < K; ++k) a = a + lut_code(lut, p.codes[k][un.start + i], lane4) * p.scales[k][un.block];
                return mean_of(a);
            };
            auto mean_quad = [&](uint32_t q) {
                v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
                if (local) {
                    const v4f l = ldg<NT>(reinterpret_cast<const v4f *>(local + un.start) + q);
                    a.x = a.x + l.x;
                    a.y = a.y + l.y;
                    a.z = a.z + l.z;
                    a.w = a.w + l.w;
                }
                for (int k = 0; k < K; ++k) {
                    const uint32_t ww = ldg<NT>(reinterpret_cast<const uint32_t *>(p.codes[k] + un.start) + q);
                    const float s = p.scales[k][un.block];
                    a.x = a.x + lut_at<0>(lut, ww, lane4) * s;
                    a.y = a.y + lut_at<1>(lut, ww, lane4) * s;
                    a.z = a.z + lut_at<2>(lut, ww, lane4) * s;
                    a.w = a.w + lut_at<3>(lut, ww, lane4) * s;
                }
                a.x = mean_of(a.x);
                a.y = mean_of(a.y);
                a.z = mean_of(a.z);
                a.w = mean_of(a.w);
                return a;
            };
            if (mean_out) {
                v4f *o4 = reinterpret_cast<v4f *>(mean_out + un.start);
                for (uint32_t q = lane; q < nq; q += kWave) stg<NT>(o4 + q, mean_quad(q));
                for (uint32_t i = done + lane; i < un.len; i += kWave) mean_out[un.start + i] = mean_at(i);
            }
            if (codes_out) {
                float fm = 0.0f;
                for (uint32_t q = lane; q < nq; q += kWave) fm = max4_abs(mean_quad(q), fm);
                uint32_t m = f2u(fm);
                for (uint32_t i = done + lane; i < un.len; i += kWave) {
                    const uint32_t a = abs_bits(mean_at(i));
                    m = m > a ? m : a;
                }
                const float s = u2f(wave_max_u32(m));
                if (lane == 0) scales_out[un.block] = s;
                const float d = s == 0.0f ? 1.0f : s;
                const float r = 1.0f / d;
                const bool recip = reciprocal_ok(d);
                uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out + un.start);
                for (uint32_t q = lane; q < nq; q += kWave) stg<1>(c4 + q, encode_quad<FASTDIV>(sr, mean_quad(q), d, r, recip));
                for (uint32_t i = done + lane; i < un.len; i += kWave)
                    codes_out[un.start + i] = (uint8_t)encode_one<FASTDIV>(sr, mean_at(i), d, r, recip);
            }
        }
    }
}

// The same average-then-compress round for K = 2, 4 or 8 workers at full speed.  A team of four
// wavefronts owns a unit of 4096 elements (one scale block): every lane holds four quads of
// running sums and K x 4 code words.  The code words are one register set that is refilled
// in place: as soon as worker k's words of the current unit have been decoded and added, the
// loads of worker k's words of the team's next unit are issued into the same registers, so
// loads are in flight all through the reduction to the block maximum (wave reduction, then one
// LDS exchange between the team's wavefronts) and the compression from the registers.
// TEAMS teams share a workgroup and its tables; the workgroup barrier that separates the
// exchange of the maxima from their use is executed by every wavefront the same number of
// times (`iters`), whether or not its team still has a unit.
// RAGGED = true (chosen by the host for blocks shorter than 4096): a unit of fewer whole aligned quads
// takes the register path as well.
template <int KT, int NT, bool FASTDIV, int TEAMS, bool RAGGED>
struct AvgTeam {
    static constexpr int Q = kUnitQuads / kWavesPerWg;  // 4 quads per lane

    WorkerPtrs p;
    const float *local;
    float *scales_out;
    uint8_t *codes_out;
    size_t n, B, nb, n_units;
    const float *lut;
    uint32_t *slots;
    Search sr;
    uint32_t lane4, lane, team, wv, tl, phase;
    float fk, rk;
    bool pow2;
    uint32_t w[KT][Q];  // code words: of the current unit until used, then of the next one

    struct Slot {
        Unit un;
        bool active, fast;
    };

    __device__ __forceinline__ float mean_of(float acc) const { return pow2 ? acc * rk : acc / fk; }

    // Element i of the unit, the slow way.
    __device__ __forceinline__ float mean_at(const Unit &un, uint32_t i) const
    {
        float a = 0.0f;
        if (local) a = a + local[un.start + i];
#pragma unroll
        for (int k = 0; k < KT; ++k) a = a + lut_code(lut, p.codes[k][un.start + i], lane4) * p.scales[k][un.block];
        return mean_of(a);
    }

    // Geometry of unit u and whether it can take the register path.
    __device__ __forceinline__ void open(size_t u, Slot &sl) const
    {
        sl.active = u < n_units;
        sl.fast = false;
        if (!sl.active) return;
        sl.un = unit_of<kUnit>(u, n, B, nb, 1);
        // whole aligned quads: a short unit takes the register path too (see load_worker)
        bool f = (RAGGED ? (sl.un.len >= 4 && (sl.un.len & 3) == 0) : sl.un.len == kUnit) &&
                 (((uintptr_t)(codes_out + sl.un.start) & 3) == 0);
#pragma unroll
        for (int k = 0; k < KT; ++k) f = f && (((uintptr_t)(p.codes[k] + sl.un.start) & 3) == 0);
        if (local) f = f && (((uintptr_t)(local + sl.un.start) & 15) == 0);
        sl.fast = f;
    }

    // This lane's j-th quad of the unit; WHOLE promises a unit of 4096 elements, otherwise a quad past the
    // end of a shorter unit becomes the unit's last one (an unconditional load of valid memory whose result
    // is not stored and cannot change the maximum).
    template <bool WHOLE>
    __device__ __forceinline__ uint32_t quad_of(const Slot &sl, int j) const
    {
        const uint32_t i = j * kWg + tl;
        if (WHOLE || !RAGGED) return i;
        const uint32_t last = (sl.un.len >> 2) - 1;
        return i < last ? i : last;
    }

    template <bool WHOLE>
    __device__ __forceinline__ void load_worker(const Slot &sl, int k)
    {
        const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k] + sl.un.start);
#pragma unroll
        for (int j = 0; j < Q; ++j) w[k][j] = ldg_at<NT>(c4, quad_of<WHOLE>(sl, j));
    }

    __device__ __forceinline__ void load_all(const Slot &sl)
    {
        if (sl.fast) {
#pragma unroll
            for (int k = 0; k < KT; ++k) load_worker<false>(sl, k);
        }
    }

    // Processes unit `sl`, whose code words are in w if it is fast, and leaves the words of `nx` there.
    // STEADY: the caller knows that both units exist and are whole and aligned (true for all but a
    // team's last two units when the host found the buffers aligned), so nothing here is
    // conditional and the compiler waits for exactly the loads each step needs.
    template <bool STEADY>
    __device__ __forceinline__ void process(const Slot &sl, const Slot &nx)
    {
        v4f acc[Q];
        uint32_t m = 0;
        if (STEADY || (sl.active && sl.fast)) {
            if (local) {  // not prefetched: the code words take the registers
                const v4f *l4 = reinterpret_cast<const v4f *>(local + sl.un.start);
#pragma unroll
                for (int j = 0; j < Q; ++j) {  // the sum starts at +0: a local -0 becomes +0
                    const v4f l = ldg<NT>(l4 + quad_of<STEADY>(sl, j));
                    acc[j].x = 0.0f + l.x;
                    acc[j].y = 0.0f + l.y;
                    acc[j].z = 0.0f + l.z;
                    acc[j].w = 0.0f + l.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < Q; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
            }
            float sc[KT];  // the K scales of this block, moved to scalar registers
#pragma unroll
            for (int k = 0; k < KT; ++k) sc[k] = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(p.scales[k][sl.un.block])));
#pragma unroll
            for (int k = 0; k < KT; ++k) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    acc[j].x = acc[j].x + lut_at<0>(lut, w[k][j], lane4) * sc[k];
                    acc[j].y = acc[j].y + lut_at<1>(lut, w[k][j], lane4) * sc[k];
                    acc[j].z = acc[j].z + lut_at<2>(lut, w[k][j], lane4) * sc[k];
                    acc[j].w = acc[j].w + lut_at<3>(lut, w[k][j], lane4) * sc[k];
                }
                // Pin the sums here.  Otherwise the compiler starts the lookups of every worker
                // at once and holds all K x 16 products in registers until the ordered sums get
                // to them, which costs a wavefront per SIMD.
#pragma unroll
                for (int j = 0; j < Q; ++j) asm volatile("" : "+v"(acc[j].x), "+v"(acc[j].y), "+v"(acc[j].z), "+v"(acc[j].w));
                if (STEADY || nx.fast) load_worker<STEADY>(nx, k);  // refill in place
            }
            float fm = 0.0f;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                acc[j].x = mean_of(acc[j].x);
                acc[j].y = mean_of(acc[j].y);
                acc[j].z = mean_of(acc[j].z);
                acc[j].w = mean_of(acc[j].w);
                fm = max4_abs(acc[j], fm);
            }
            m = f2u(fm);
        } else {
            if (sl.active) {
                for (uint32_t i = tl; i < sl.un.len; i += kWg) {
                    const uint32_t a = abs_bits(mean_at(sl.un, i));
                    m = m > a ? m : a;
                }
            }
            load_all(nx);
        }
        m = wave_max_u32(m);
        uint32_t *sp = slots + (phase * TEAMS + team) * kWavesPerWg;
        if (lane == 0) sp[wv] = m;
        __syncthreads();
        {
            const uint32_t a = sp[0] > sp[1] ? sp[0] : sp[1], b = sp[2] > sp[3] ? sp[2] : sp[3];
            m = (uint32_t)__builtin_amdgcn_readfirstlane((int)(a > b ? a : b));
        }
        phase ^= 1;  // the other half of the slots next time: one barrier per unit is enough
        if (!STEADY && !sl.active) return;
        const float s = u2f(m);
        if (tl == 0) scales_out[sl.un.block] = s;
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        if (STEADY || sl.fast) {
            uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out + sl.un.start);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const uint32_t cw = encode_quad<FASTDIV>(sr, acc[j], d, r, recip);
                if (STEADY || !RAGGED || j * kWg + tl < (sl.un.len >> 2)) stg<1>(c4 + j * kWg + tl, cw);
            }
        } else {
            for (uint32_t i = tl; i < sl.un.len; i += kWg)
                codes_out[sl.un.start + i] = (uint8_t)encode_one<FASTDIV>(sr, mean_at(sl.un, i), d, r, recip);
        }
    }
};

template <int KT, int NT, bool FASTDIV, int TEAMS, bool REMAP, bool RAGGED>
__global__ __launch_bounds__(kWg * TEAMS, TEAMS == 3 ? 3 : 4) void k_avg_team(const uint32_t *__restrict__ tab, WorkerPtrs p,
                                                            const float *__restrict__ local, size_t n, size_t B, size_t nb,
                                                            size_t n_units, size_t n_teams, uint32_t iters, uint32_t steady,
                                                            float *__restrict__ scales_out, uint8_t *__restrict__ codes_out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t dyn_lds[];  // 2 phases x TEAMS x 4 maxima, then the bucket table
    constexpr int kSlots = 2 * TEAMS * kWavesPerWg;
    using Avg = AvgTeam<KT, NT, FASTDIV, TEAMS, RAGGED>;
    Avg e;
    e.p = p;
    e.local = local;
    e.scales_out = scales_out;
    e.codes_out = codes_out;
    e.n = n;
    e.B = B;
    e.nb = nb;
    e.n_units = n_units;
    e.lut = lut;
    e.slots = dyn_lds;
    e.lane = threadIdx.x & 63;
    e.lane4 = e.lane * 4;
    const uint32_t wave = wave_in_wg();
    e.team = wave / kWavesPerWg;
    e.wv = wave % kWavesPerWg;
    e.tl = threadIdx.x & (kWg - 1);  // lane within the team
    e.phase = 0;
    const int terms = KT + (local ? 1 : 0);
    e.fk = (float)terms;
    e.rk = 1.0f / e.fk;
    e.pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    size_t u = (size_t)blockIdx.x * TEAMS + e.team;
    typename Avg::Slot a, b;
    e.open(u, a);
    e.load_all(a);  // the first loads are in flight while the tables are copied
    load_lut(tab, lut);
    {
        e.sr = load_bucket_table(tab, dyn_lds + kSlots, kWg * TEAMS);
        if (!REMAP) e.sr.remap = nullptr;  // a type without a rank-to-code table: no test for one in the loop
    }
    __syncthreads();
    // `steady` (even) leading iterations in which this and the next unit of every team are whole
    // aligned units, then the general ones.
    uint32_t it = 0;
    for (; it < steady; it += 2) {
        e.open(u + n_teams, b);
        e.template process<true>(a, b);
        u += n_teams;
        e.open(u + n_teams, a);
        e.template process<true>(b, a);
        u += n_teams;
    }
    for (; it < iters; it += 2) {
        e.open(u + n_teams, b);
        e.template process<false>(a, b);
        u += n_teams;
        if (it + 1 >= iters) break;
        e.open(u + n_teams, a);
        e.template process<false>(b, a);
        u += n_teams;
    }
}

// Approximation-error statistics of compress-then-decompress (Sec. 3.4, Table 2).  Per block b,
// stats[4 b + 0] = sum of e, [1] = sum of e / |x| over x != 0, [2] = number of x != 0,
// [3] = largest e, with q = fl32(cb[code] * s) and e = |(double) q - (double) x| (one binary64
// subtraction; the quotient one correctly rounded binary64 division).  stats[] was zeroed.
// A wavefront walks a contiguous run of units of Q * 256 elements, keeps binary64 running sums per
// lane while the block stays the same, and merges them into stats[] with atomics when the block
// changes and at the end: the count and the maximum are exact in any order (integers below 2^53,
// and non-negative binary64 numbers order like their bit patterns); the two sums depend on the
// order only in their last bits.
template <int Q>
__global__ __launch_bounds__(kWg) void k_error_stats(const uint32_t *__restrict__ tab, const float *__restrict__ x, size_t n,
                                                    size_t B, size_t nb, size_t upb, size_t n_units, size_t per_wave,
                                                    const float *__restrict__ scales, double *__restrict__ stats)
{
    constexpr int U = Q * 4 * kWave;
    extern __shared__ uint32_t lds[];  // 256 table values, then the search tables
    for (uint32_t i = threadIdx.x; i < 256; i += kWg) lds[i] = tab[kCbOff + i];
    const Search sr = load_bucket_table(tab, lds + 256);
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    const size_t u0 = first_unit() * per_wave;
    const size_t u1 = u0 + per_wave < n_units ? u0 + per_wave : n_units;
    double sum_abs = 0.0, sum_rel = 0.0, count = 0.0, worst = 0.0;
    auto add = [&](float xv, uint32_t code, float s) {
        const float q = u2f(lds[code & 0xFFu]) * s;
        const double e = __builtin_fabs((double)q - (double)xv);
        const double rel = e / __builtin_fabs((double)xv);  // not used when xv is a zero
        sum_abs += e;
        sum_rel += xv != 0.0f ? rel : 0.0;
        count += xv != 0.0f ? 1.0 : 0.0;
        worst = e > worst ? e : worst;
    };
    auto flush = [&](size_t blk) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {  // the same tree in every launch
            sum_abs += __shfl_xor(sum_abs, m);
            sum_rel += __shfl_xor(sum_rel, m);
            count += __shfl_xor(count, m);
            const double o = __shfl_xor(worst, m);
            worst = o > worst ? o : worst;
        }
        if (lane == 0) {
            double *p = stats + 4 * blk;
            atomicAdd(p, sum_abs);
            atomicAdd(p + 1, sum_rel);
            atomicAdd(p + 2, count);
            atomicMax(reinterpret_cast<unsigned long long *>(p + 3), (unsigned long long)__double_as_longlong(worst));
        }
        sum_abs = sum_rel = count = worst = 0.0;
    };
    bool open = false;
    size_t cur = 0;
    for (size_t u = u0; u < u1; ++u) {
        const Unit un = unit_of<U>(u, n, B, nb, upb);
        if (open && un.block != cur) flush(cur);
        open = true;
        cur = un.block;
        const float s = scales[un.block];
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        const float *px = x + un.start;
        if (un.len == U && ((uintptr_t)px & 15) == 0) {
            const v4f *p4 = reinterpret_cast<const v4f *>(px);
            v4f v[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) v[j] = ldg<1>(p4 + j * kWave + lane);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const uint32_t c = encode_quad<true>(sr, v[j], d, r, recip);
                add(v[j].x, c, s);
                add(v[j].y, c >> 8, s);
                add(v[j].z, c >> 16, s);
                add(v[j].w, c >> 24, s);
            }
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) add(px[i], encode_one<true>(sr, px[i], d, r, recip), s);
        }
    }
    if (open) flush(cur);
}

// Means over all blocks from the per-block statistics: means[0] = (sum of absolute errors) / n,
// means[1] = (sum of relative errors) / (number of non-zero inputs), 0 when there is none.
// One workgroup of 1024 threads; thread t adds blocks t, t + 1024, ... in that order and the threads'
// sums are combined by a fixed tree, so the result is the same in every launch.
constexpr uint32_t kMeansThreads = 1024;
__global__ __launch_bounds__(kMeansThreads) void k_error_means(const double *__restrict__ stats, size_t nb, size_t n,
                                                              double *__restrict__ means)
{
    __shared__ double part[3][kMeansThreads];
    double a = 0.0, r = 0.0, c = 0.0;
#pragma unroll 4
    for (size_t b = threadIdx.x; b < nb; b += kMeansThreads) {
        a += stats[4 * b];
        r += stats[4 * b + 1];
        c += stats[4 * b + 2];
    }
    part[0][threadIdx.x] = a;
    part[1][threadIdx.x] = r;
    part[2][threadIdx.x] = c;
    __syncthreads();
    for (uint32_t w = kMeansThreads / 2; w >= 1; w >>= 1) {
        if (threadIdx.x < w) {
            part[0][threadIdx.x] += part[0][threadIdx.x + w];
            part[1][threadIdx.x] += part[1][threadIdx.x + w];
            part[2][threadIdx.x] += part[2][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        means[0] = part[0][0] / (double)n;
        means[1] = part[2][0] > 0.0 ? part[1][0] / part[2][0] : 0.0;
    }
}

// ---------------------------------------------------------------- host side

thread_local char t_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(t_err, sizeof(t_err), fmt, ap);
    va_end(ap);
    return code;
}

#define DQ8_HIP(call)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess) return fail(DQ8_ERR_DEVICE, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)

constexpr int kMaxDevices = 64;

struct DeviceState {
    bool ready = false;
    uint32_t *tables = nullptr;  // device address of g_tables on this device
    int cus = 0;
    bool has_remap[kKinds] = {false, false, false, false};  // the type needs the rank-to-code table
    uint32_t search_words[kKinds] = {0, 0, 0, 0};  // LDS words of a type's search tables (buckets + rank-to-code)
};

std::mutex g_mu;
DeviceState g_dev[kMaxDevices];

int device_state(DeviceState **out)
{
    int dev = -1;
    DQ8_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(DQ8_ERR_DEVICE, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceState &st = g_dev[dev];
    if (!st.ready) {
        static uint32_t image[kKinds][kTableWords];
        for (int k = 0; k < kKinds; ++k) {
            static dq8::Tables t;
            int rc = dq8::build_tables(k, &t);
            if (rc) return fail(DQ8_ERR_KIND, "table construction failed for kind %d (status %d)", k, rc);
            dq8::pack_tables(t, image[k]);
            st.has_remap[k] = t.has_remap;
            st.search_words[k] = t.n_bucket + (t.has_remap ? (uint32_t)kRemapWords : 0u);
        }
        void *sym = nullptr;
        DQ8_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(g_tables)));
        DQ8_HIP(hipMemcpy(sym, image, sizeof(image), hipMemcpyHostToDevice));
        hipDeviceProp_t prop;
        DQ8_HIP(hipGetDeviceProperties(&prop, dev));
        st.tables = static_cast<uint32_t *>(sym);
        st.cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        st.ready = true;
    }
    *out = &st;
    return DQ8_OK;
}

// Launch shape of each kernel.  Defaults come from measurements on MI355X (bandwidth peaks
// at roughly 16-32 KiB of loads in flight per compute unit); dq8_internal_tune() changes them
// for experiments.  None of them affects results.
struct Tuning {
    int amax_nt = 1;     // cache policy of each kernel's streaming accesses, see ldg / stg
    int avg_lean = 1;    // decode-and-average of whole aligned units: the kernel without slow paths in its loop
    int avg_lean_q = 2;  //   its code words per lane and worker, wavefronts per compute unit and per workgroup
    int avg_lean_wpc = 4;
    int avg_lean_wpw = 4;
    int copy_nt = 1;
    int fastdiv = 1;     // reciprocal multiply with exact fallback near thresholds
    int enc_wpb = 4;     // wavefronts per unit in the encoder: 1 or 4
    int enc_wpc = 24;    // encoder wavefronts per compute unit (general kernel)
    int enc_lean = 1;    // whole aligned 4096-element blocks go to the kernel without slow paths in its loop,
    int enc_lean_wpc = 8;  //   which keeps its loads in flight with this many wavefronts per compute unit
    int enc_fill = 1;    //   and puts a team on every resident slot, even if some then get one block fewer
    int amax_q = 16;     // absmax: quads per lane in flight (unit = 256 q elements)
    int amax_wpc = 4;
    int dec_q = 16;      // decode: code words per lane in flight
    int dec_wpc = 4;
    int dec_wpw = 4;     // decode: wavefronts per workgroup (they share one table in LDS)
    int avg_q = 2;       // decode-and-average: code words per lane and worker in flight
    int avg_wpc = 32;
    int avg_wpw = 16;
    int blk_wpw = 8;     // register-resident average: wavefronts per workgroup (two workgroups per compute unit)
    int avg_team = 1;    // average-then-compress with K = 2, 4, 8: the team kernel (0: the wave-per-block kernel)
    int avg_steady = 1;  //   unconditional steady-state iterations when the buffers are aligned
    int avg_teams = 3;   //   teams per workgroup: 2, 3 or 4
    int avg_wgpc = 1;    //   workgroups per compute unit (2 only with 2 teams)
    int copy_q = 2;
    int copy_wpc = 8;
};
Tuning g_tune;

struct Plan {
    size_t B, nb, upb, n_units, n_teams;
    unsigned grid;
};

// Units, and a grid in which every team (wpb wavefronts) walks the same number of them.
Plan make_plan(size_t n, size_t block, int cus, int waves_per_cu, int wpb, int waves_per_wg = kWavesPerWg,
               size_t unit = kUnit)
{
    Plan p;
    p.B = (block == 0 || block > n) ? n : block;
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

bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

int check_kind(int kind)
{
    if (kind < 0 || kind >= kKinds) return fail(DQ8_ERR_KIND, "unknown data type %d", kind);
    return DQ8_OK;
}

int after_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DQ8_ERR_DEVICE, "launch of %s failed: %s", what, hipGetErrorString(e));
    return DQ8_OK;
}

int launch_absmax(const DeviceState &st, const float *x, size_t n, size_t block, float *scales, hipStream_t stream)
{
    // Units no longer than a block (so that whole blocks are whole units when the block is a power of two),
    // and the more wavefronts per compute unit the smaller the unit: the bytes in flight stay the same.
    const size_t Bq = (block == 0 || block > n) ? n : block;
    int q = (g_tune.amax_q == 1 || g_tune.amax_q == 2 || g_tune.amax_q == 8 || g_tune.amax_q == 16) ? g_tune.amax_q : 4;
    int wpc = g_tune.amax_wpc;
    while (q > 1 && (size_t)q * 4 * kWave > Bq) {
        q >>= 1;
        wpc = wpc * 2 > 32 ? 32 : wpc * 2;
    }
    Plan p = make_plan(n, block, st.cus, wpc, 1, kWavesPerWg, (size_t)q * 4 * kWave);
    size_t per_wave = 0;
    if (p.upb > 1) {
        unsigned g = (unsigned)((p.nb + 255) / 256);
        hipLaunchKernelGGL(k_fill_zero, dim3(g), dim3(256), 0, stream, scales, p.nb);
        int rc = after_launch("k_fill_zero");
        if (rc) return rc;
        per_wave = (p.n_units + p.n_teams - 1) / p.n_teams;
    }
#define DQ8_AMAX(Q, NT)                                                                                          \
    hipLaunchKernelGGL((k_absmax<Q, NT>), dim3(p.grid), dim3(kWg), 0, stream, x, n, p.B, p.nb, p.upb, p.n_units, \
                       p.n_teams, per_wave, scales)
#define DQ8_AMAX_Q(NT)                      \
    switch (q) {                            \
    case 1: DQ8_AMAX(1, NT); break;         \
    case 2: DQ8_AMAX(2, NT); break;         \
    case 8: DQ8_AMAX(8, NT); break;         \
    case 16: DQ8_AMAX(16, NT); break;       \
    default: DQ8_AMAX(4, NT); break;        \
    }
    if (g_tune.amax_nt) {
        DQ8_AMAX_Q(1)
    } else {
        DQ8_AMAX_Q(0)
    }
#undef DQ8_AMAX_Q
#undef DQ8_AMAX
    return after_launch("k_absmax");
}

int launch_encode(const DeviceState &st, int kind, const float *x, size_t n, size_t block, float *scales, uint8_t *codes,
                  bool fused, hipStream_t stream)
{
    // Unit = the smallest power of two that holds a block, between 256 and 4096 elements.  4096: a team of four
    // wavefronts per unit, four quads per lane.  Smaller: one wavefront per unit (1, 2, 4 or 8 quads per lane) and
    // every wavefront slot of the compute units in use.
    const size_t Bq = (block == 0 || block > n) ? n : block;
    size_t unit = 256;
    while (unit < Bq && unit < (size_t)kUnit) unit <<= 1;
    const bool small = unit < (size_t)kUnit;
    const int wpb = small ? 1 : (g_tune.enc_wpb == 4 ? 4 : 1);
    const int ql = (int)(unit / (size_t)(4 * kWave * wpb));
    Plan p = make_plan(n, block, st.cus, small ? 32 : g_tune.enc_wpc, wpb, kWavesPerWg, unit);
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = ((size_t)st.search_words[kind] + kTeamSlots) * sizeof(uint32_t);
    // Whole aligned blocks of exactly one unit: the kernel without slow paths in its loop.
    if (fused && g_tune.enc_lean && p.B == (size_t)kUnit && n / kUnit >= 1 && n / kUnit < 0xFFFFFFFFull &&
        ((uintptr_t)x & 15) == 0 && ((uintptr_t)codes & 3) == 0) {
        const uint32_t n_full = (uint32_t)(n / kUnit), tail = (uint32_t)(n % kUnit);
        size_t teams = (size_t)st.cus * (size_t)g_tune.enc_lean_wpc / 4;  // a team on every resident slot
        if (!g_tune.enc_fill) {  // or the smaller grid in which no team gets a block fewer than another
            const size_t per = (n_full + teams - 1) / teams;
            teams = (n_full + per - 1) / per;
        }
        if (teams > n_full) teams = n_full;
#define DQ8_ENC_FULL(FD, RM)                                                                                        \
    hipLaunchKernelGGL((k_encode_full<1, FD, RM>), dim3((unsigned)teams), dim3(kWg), lds, stream, tab, x, n_full, \
                       (uint32_t)teams, tail, scales, codes)
        if (st.has_remap[kind]) {
            DQ8_ENC_FULL(true, true);
        } else if (g_tune.fastdiv) {
            DQ8_ENC_FULL(true, false);
        } else {
            DQ8_ENC_FULL(false, false);
        }
#undef DQ8_ENC_FULL
        return after_launch("k_encode_full");
    }
#define DQ8_ENC(WPB, QL, FUSED, FD)                                                                               \
    hipLaunchKernelGGL((k_encode<WPB, QL, 1, FUSED, FD>), dim3(p.grid), dim3(kWg), lds, stream, tab, x, n, p.B, p.nb, \
                       p.upb, p.n_units, p.n_teams, scales, codes)
#define DQ8_ENC_F(WPB, QL, FD)       \
    if (fused) {                     \
        DQ8_ENC(WPB, QL, true, FD);  \
    } else {                         \
        DQ8_ENC(WPB, QL, false, FD); \
    }
    const bool fd = g_tune.fastdiv != 0;
    if (wpb == 4) {
        if (fd) {
            DQ8_ENC_F(4, 4, true)
        } else {
            DQ8_ENC_F(4, 4, false)
        }
    } else {
        switch (ql) {
        case 1: DQ8_ENC_F(1, 1, true) break;
        case 2: DQ8_ENC_F(1, 2, true) break;
        case 4: DQ8_ENC_F(1, 4, true) break;
        case 8: DQ8_ENC_F(1, 8, true) break;
        default:
            if (fd) {
                DQ8_ENC_F(1, 16, true)
            } else {
                DQ8_ENC_F(1, 16, false)
            }
            break;
        }
    }
#undef DQ8_ENC_F
#undef DQ8_ENC
    return after_launch("k_encode");
}

// Error statistics of compress-then-decompress into stats[4 nb] (and means[2] when not NULL).
int launch_error_stats(const DeviceState &st, int kind, const float *x, size_t n, size_t block, const float *scales,
                       double *stats, double *means, hipStream_t stream)
{
    constexpr int Q = 4;
    Plan p = make_plan(n, block, st.cus, 16, 1, kWavesPerWg, (size_t)Q * 4 * kWave);
    const size_t zero_words = 8 * p.nb;  // 4 binary64 zeros per block
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<float *>(stats), zero_words);
    int rc = after_launch("k_fill_zero");
    if (rc) return rc;
    const size_t per_wave = (p.n_units + p.n_teams - 1) / p.n_teams;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = (256 + (size_t)st.search_words[kind]) * sizeof(uint32_t);
    hipLaunchKernelGGL((k_error_stats<Q>), dim3(p.grid), dim3(kWg), lds, stream, tab, x, n, p.B, p.nb, p.upb, p.n_units,
                       per_wave, scales, stats);
    rc = after_launch("k_error_stats");
    if (rc || !means) return rc;
    hipLaunchKernelGGL(k_error_means, dim3(1), dim3(kMeansThreads), 0, stream, stats, p.nb, n, means);
    return after_launch("k_error_means");
}

// Copies and checks the K (codes, scales) pairs of a call; `out` / `out_bytes` is a buffer the
// call writes that must not overlap any of them (may be NULL).
int gather_workers(const char *who, const uint8_t *const *codes, const float *const *scales, int K, size_t n, size_t nb,
                   const void *out, size_t out_bytes, WorkerPtrs *wp)
{
    std::memset(wp, 0, sizeof(*wp));
    if (K > 0 && (!codes || !scales)) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    for (int k = 0; k < K; ++k) {
        if (!codes[k] || !scales[k]) return fail(DQ8_ERR_NULL, "%s: worker %d has a NULL buffer", who, k);
        if (out && (overlaps(out, out_bytes, codes[k], n) || overlaps(out, out_bytes, scales[k], nb * 4)))
            return fail(DQ8_ERR_ARG, "%s: an output overlaps worker %d", who, k);
        wp->codes[k] = codes[k];
        wp->scales[k] = scales[k];
    }
    return DQ8_OK;
}

// Average-then-compress for K = 2, 4, 8: teams of four wavefronts; two teams per workgroup and two
// workgroups per compute unit (128 registers per lane), or three teams in one workgroup per compute
// unit (170 registers per lane).
int launch_avg_team(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                    size_t block, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    const size_t Bq = (block == 0 || block > n) ? n : block;
    const bool ragged = Bq != (size_t)kUnit;  // shorter blocks: the variant whose register path takes short units
    const int teams = ragged ? 3 : ((g_tune.avg_teams == 3 || g_tune.avg_teams == 4) ? g_tune.avg_teams : 2);
    const int wgs_per_cu = (teams == 2 && g_tune.avg_wgpc == 2) ? 2 : 1;
    Plan p = make_plan(n, block, st.cus, 4 * teams * wgs_per_cu, 4, 4 * teams, kUnit);
    const uint32_t iters = (uint32_t)((p.n_units + p.n_teams - 1) / p.n_teams);
    // Iterations in which every team's current and next unit are whole aligned blocks.
    uint32_t steady = 0;
    bool aligned = g_tune.avg_steady && p.B == (size_t)kUnit && ((uintptr_t)codes_out & 3) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) aligned = aligned && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (aligned) {
        const size_t all_valid = (n / kUnit) / p.n_teams;  // iterations in which every team has a whole unit
        if (all_valid >= 2) steady = (uint32_t)((all_valid - 1) & ~(size_t)1);
    }
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = ((size_t)st.search_words[kind] + 2 * teams * kWavesPerWg) * sizeof(uint32_t);
#define DQ8_TEAM(KT, RM, T, RG)                                                                                          \
    hipLaunchKernelGGL((k_avg_team<KT, 1, true, T, RM, RG>), dim3(p.grid), dim3(kWg * T), lds, stream, tab, wp, local, n, \
                       p.B, p.nb, p.n_units, p.n_teams, iters, steady, scales_out, codes_out)
#define DQ8_TEAM_T(KT, RM)              \
    if (ragged) {                       \
        DQ8_TEAM(KT, RM, 3, true);      \
    } else if (teams == 3) {            \
        DQ8_TEAM(KT, RM, 3, false);     \
    } else if (teams == 4) {            \
        DQ8_TEAM(KT, RM, 4, false);     \
    } else {                            \
        DQ8_TEAM(KT, RM, 2, false);     \
    }
#define DQ8_TEAM_RM(KT)          \
    if (st.has_remap[kind]) {    \
        DQ8_TEAM_T(KT, true)     \
    } else {                     \
        DQ8_TEAM_T(KT, false)    \
    }
    switch (K) {
    case 2: DQ8_TEAM_RM(2) break;
    case 4: DQ8_TEAM_RM(4) break;
    default: DQ8_TEAM_RM(8) break;
    }
#undef DQ8_TEAM_RM
#undef DQ8_TEAM_T
#undef DQ8_TEAM
    return after_launch("k_avg_team");
}

int launch_avg_block(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                     size_t block, float *mean_out, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    // Unit = the smallest power of two that holds a block, between 256 and 4096 elements.
    const size_t Bq = (block == 0 || block > n) ? n : block;
    size_t unit = 256;
    while (unit < Bq && unit < (size_t)kUnit) unit <<= 1;
    // K = 2, 4, 8 and blocks that need a 4096-element unit: the team kernel
    if (codes_out && !mean_out && (K == 2 || K == 4 || K == 8) && g_tune.avg_team && unit == (size_t)kUnit)
        return launch_avg_team(st, kind, wp, K, local, n, block, scales_out, codes_out, stream);
    const int ql = (int)(unit / (size_t)(4 * kWave));
    // whole 4096-element units with short ends need the 170 registers per lane that six wavefronts leave
    const bool ragged = Bq < n && Bq % unit != 0;  // blocks end inside units
    const int wpw = (ql == 16 && (ragged || g_tune.blk_wpw != 8)) ? 6 : 8;
    Plan p = make_plan(n, block, st.cus, 2 * wpw, 1, wpw, unit);
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = codes_out ? (size_t)st.search_words[kind] * sizeof(uint32_t) : 0;
#define DQ8_BLK(QL, WPW, RG)                                                                                              \
    hipLaunchKernelGGL((k_avg_block<QL, 2, true, WPW, RG>), dim3(p.grid), dim3(kWave * WPW), lds, stream, tab, wp, K, local, \
                       n, p.B, p.nb, p.upb, p.n_units, p.n_teams, mean_out, scales_out, codes_out)
#define DQ8_BLK_R(QL, WPW)       \
    if (ragged) {                \
        DQ8_BLK(QL, WPW, true);  \
    } else {                     \
        DQ8_BLK(QL, WPW, false); \
    }
    switch (ql) {
    case 1: DQ8_BLK_R(1, 8) break;
    case 2: DQ8_BLK_R(2, 8) break;
    case 4: DQ8_BLK_R(4, 8) break;
    case 8: DQ8_BLK_R(8, 8) break;
    default:
        if (wpw == 8) {
            DQ8_BLK_R(16, 8)
        } else {
            DQ8_BLK_R(16, 6)
        }
        break;
    }
#undef DQ8_BLK_R
#undef DQ8_BLK
    return after_launch("k_avg_block");
}

// K-way decode-and-average (K = 2, 4, 8; optional local term) of whole aligned units with a power-of-two
// number of them per block (or a single block): the kernel without slow paths in its loop.
// *launched = false (and nothing done) when the buffers do not qualify.
int launch_avg_full(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                    const Plan &p, float *out, hipStream_t stream, bool *launched)
{
    *launched = false;
    const int lq = g_tune.avg_lean_q == 4 ? 4 : 2;
    const int lw = g_tune.avg_lean_wpw == 16 ? 16 : (g_tune.avg_lean_wpw == 8 ? 8 : 4);
    const size_t U = (size_t)lq * 4 * kWave;
    const size_t upb_l = p.B / U;
    bool ok = p.nb == 1 || (p.B % U == 0 && (upb_l & (upb_l - 1)) == 0);
    ok = ok && n / U >= 1 && n / U < 0x7FFFFFFFull && ((uintptr_t)out & 15) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) ok = ok && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (!ok) return DQ8_OK;
    uint32_t shift = 31;  // a single block: every unit belongs to block 0
    if (p.nb > 1) {
        shift = 0;
        while (((size_t)1 << shift) < upb_l) ++shift;
    }
    const uint32_t n_full = (uint32_t)(n / U), tail = (uint32_t)(n % U);
    size_t waves = (size_t)st.cus * (size_t)g_tune.avg_lean_wpc;
    if (waves > n_full) waves = n_full;
    const unsigned grid = (unsigned)((waves + lw - 1) / lw);
    const uint32_t n_waves = grid * (uint32_t)lw;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
#define DQ8_AVGL(KT, Q, WPW, LOC)                                                                                     \
    hipLaunchKernelGGL((k_decode_avg_full<KT, Q, 2, WPW, LOC>), dim3(grid), dim3(kWave * WPW), 0, stream, tab, wp, local, \
                       n_full, n_waves, shift, tail, out)
#define DQ8_AVGL_L(KT, Q, WPW)         \
    if (local) {                       \
        DQ8_AVGL(KT, Q, WPW, true);    \
    } else {                           \
        DQ8_AVGL(KT, Q, WPW, false);   \
    }
#define DQ8_AVGL_W(KT, Q)                  \
    switch (lw) {                          \
    case 16: DQ8_AVGL_L(KT, Q, 16) break;  \
    case 8: DQ8_AVGL_L(KT, Q, 8) break;    \
    default: DQ8_AVGL_L(KT, Q, 4) break;   \
    }
#define DQ8_AVGL_Q(KT)                     \
    if (lq == 4) {                         \
        DQ8_AVGL_W(KT, 4)                  \
    } else {                               \
        DQ8_AVGL_W(KT, 2)                  \
    }
    switch (K) {
    case 2: DQ8_AVGL_Q(2) break;
    case 4: DQ8_AVGL_Q(4) break;
    default: DQ8_AVGL_Q(8) break;
    }
#undef DQ8_AVGL_Q
#undef DQ8_AVGL_W
#undef DQ8_AVGL_L
#undef DQ8_AVGL
    *launched = true;
    return after_launch("k_decode_avg_full");
}

}  // namespace

extern "C" {

const char *dq8_last_error(void) { return t_err; }

int dq8_codebook(int kind, float *cb256_host)
{
    if (!cb256_host) return fail(DQ8_ERR_NULL, "dq8_codebook: cb256_host is NULL");
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    std::memcpy(cb256_host, t.cb, sizeof(t.cb));
    return DQ8_OK;
}

int dq8_init(void)
{
    DeviceState *st;
    return device_state(&st);
}

int dq8_absmax(const float *x, size_t n, size_t block, float *scales, void *hip_stream)
{
    if (n == 0) return DQ8_OK;
    if (!x || !scales) return fail(DQ8_ERR_NULL, "dq8_absmax: NULL pointer");
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "dq8_absmax: n too large");
    DeviceState *st;
    int rc = device_state(&st);
    if (rc) return rc;
    return launch_absmax(*st, x, n, block, scales, static_cast<hipStream_t>(hip_stream));
}

int dq8_encode(int kind, const float *x, size_t n, size_t block, float *scales, uint8_t *codes, unsigned flags,
               void *hip_stream)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    if (flags & ~DQ8_SCALES_GIVEN) return fail(DQ8_ERR_ARG, "dq8_encode: unknown flags 0x%x", flags);
    if (n == 0) return DQ8_OK;
    if (!x || !scales || !codes) return fail(DQ8_ERR_NULL, "dq8_encode: NULL pointer");
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "dq8_encode: n too large");
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    const size_t Bq = (block == 0 || block > n) ? n : block;
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(x, n * 4, codes, n) || overlaps(x, n * 4, scales, nbq * 4) || overlaps(codes, n, scales, nbq * 4))
        return fail(DQ8_ERR_ARG, "dq8_encode: buffers overlap");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool given = (flags & DQ8_SCALES_GIVEN) != 0;
    const bool fused = !given && Bq <= (size_t)kUnit;  // the block fits one unit: absmax and encode in one kernel
    if (!given && !fused) {
        rc = launch_absmax(*st, x, n, block, scales, stream);
        if (rc) return rc;
    }
    return launch_encode(*st, kind, x, n, block, scales, codes, fused, stream);
}

int dq8_decode(int kind, const uint8_t *codes, const float *scales, size_t n, size_t block, float *out,
               void *hip_stream)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    if (n == 0) return DQ8_OK;
    if (!codes || !scales || !out) return fail(DQ8_ERR_NULL, "dq8_decode: NULL pointer");
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "dq8_decode: n too large");
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    // Units no longer than a block, and the smaller the unit the more wavefronts per compute unit (the bytes
    // in flight stay the same); 16 wavefronts share a workgroup's 64 KiB table when there are that many.
    const size_t Bq = (block == 0 || block > n) ? n : block;
    int q = (g_tune.dec_q == 1 || g_tune.dec_q == 2 || g_tune.dec_q == 4 || g_tune.dec_q == 8) ? g_tune.dec_q : 16;
    int wpc = g_tune.dec_wpc;
    while (q > 1 && (size_t)q * 4 * kWave > Bq) {
        q >>= 1;
        wpc = wpc * 2 > 32 ? 32 : wpc * 2;
    }
    const int wpw = q == 16 ? (g_tune.dec_wpw == 16 ? 16 : (g_tune.dec_wpw == 8 ? 8 : 4)) : (q == 8 ? 8 : 16);
    Plan p = make_plan(n, block, st->cus, wpc, 1, wpw, (size_t)q * 4 * kWave);
    if (overlaps(out, n * 4, codes, n) || overlaps(out, n * 4, scales, p.nb * 4))
        return fail(DQ8_ERR_ARG, "dq8_decode: out overlaps an input");
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool ragged = p.nb > 1 && p.B % ((size_t)q * 4 * kWave) != 0;  // blocks end inside units
#define DQ8_DEC(Q, WPW, RG)                                                                                          \
    hipLaunchKernelGGL((k_decode<Q, 2, WPW, RG>), dim3(p.grid), dim3(kWave * WPW), 0, stream, tab, codes, scales, n, p.B, \
                       p.nb, p.upb, p.n_units, p.n_teams, out)
#define DQ8_DEC_R(Q, WPW)        \
    if (ragged) {                \
        DQ8_DEC(Q, WPW, true);   \
    } else {                     \
        DQ8_DEC(Q, WPW, false);  \
    }
    switch (q) {
    case 1: DQ8_DEC_R(1, 16) break;
    case 2: DQ8_DEC_R(2, 16) break;
    case 4: DQ8_DEC_R(4, 16) break;
    case 8: DQ8_DEC_R(8, 8) break;
    default:
        switch (wpw) {
        case 16: DQ8_DEC_R(16, 16) break;
        case 8: DQ8_DEC_R(16, 8) break;
        default: DQ8_DEC_R(16, 4) break;
        }
        break;
    }
#undef DQ8_DEC_R
#undef DQ8_DEC
    return after_launch("k_decode");
}

int dq8_decode_accumulate_avg(int kind, const uint8_t *const *codes, const float *const *scales, int K, size_t n,
                              size_t block, float *out, void *hip_stream)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    if (K < 1 || K > DQ8_MAX_K) return fail(DQ8_ERR_ARG, "dq8_decode_accumulate_avg: K = %d outside 1..%d", K, DQ8_MAX_K);
    if (n == 0) return DQ8_OK;
    if (!codes || !scales || !out) return fail(DQ8_ERR_NULL, "dq8_decode_accumulate_avg: NULL pointer");
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "dq8_decode_accumulate_avg: n too large");
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    const int wpw = g_tune.avg_wpw == 16 ? 16 : (g_tune.avg_wpw == 8 ? 8 : 4);
    const bool fixed_k = K == 2 || K == 4 || K == 8;
    const size_t Bq = (block == 0 || block > n) ? n : block;
    int q = !fixed_k ? 1 : ((g_tune.avg_q == 1 || g_tune.avg_q == 4) ? g_tune.avg_q : 2);
    while (q > 1 && (size_t)q * 4 * kWave > Bq) q >>= 1;  // units no longer than a block
    Plan p = make_plan(n, block, st->cus, g_tune.avg_wpc, 1, wpw, (size_t)q * 4 * kWave);
    WorkerPtrs wp;
    std::memset(&wp, 0, sizeof(wp));
    for (int k = 0; k < K; ++k) {
        if (!codes[k] || !scales[k]) return fail(DQ8_ERR_NULL, "dq8_decode_accumulate_avg: worker %d has a NULL buffer", k);
        if (overlaps(out, n * 4, codes[k], n) || overlaps(out, n * 4, scales[k], p.nb * 4))
            return fail(DQ8_ERR_ARG, "dq8_decode_accumulate_avg: out overlaps worker %d", k);
        wp.codes[k] = codes[k];
        wp.scales[k] = scales[k];
    }
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (fixed_k && g_tune.avg_lean) {
        bool launched = false;
        rc = launch_avg_full(*st, kind, wp, K, nullptr, n, p, out, stream, &launched);
        if (rc || launched) return rc;
    }
#define DQ8_AVG(KT, Q, WPW)                                                                                      \
    hipLaunchKernelGGL((k_decode_avg<KT, Q, 2, WPW>), dim3(p.grid), dim3(kWave * WPW), 0, stream, tab, wp, K, n, p.B, \
                       p.nb, p.upb, p.n_units, p.n_teams, out)
#define DQ8_AVG_W(KT, Q)                 \
    switch (wpw) {                       \
    case 16: DQ8_AVG(KT, Q, 16); break;  \
    case 8: DQ8_AVG(KT, Q, 8); break;    \
    default: DQ8_AVG(KT, Q, 4); break;   \
    }
#define DQ8_AVG_Q(KT)                    \
    switch (q) {                         \
    case 1: DQ8_AVG_W(KT, 1) break;      \
    case 4: DQ8_AVG_W(KT, 4) break;      \
    default: DQ8_AVG_W(KT, 2) break;     \
    }
    switch (K) {
    case 2: DQ8_AVG_Q(2) break;
    case 4: DQ8_AVG_Q(4) break;
    case 8: DQ8_AVG_Q(8) break;
    default: DQ8_AVG_W(0, 1) break;
    }
#undef DQ8_AVG_Q
#undef DQ8_AVG_W
#undef DQ8_AVG
    return after_launch("k_decode_avg");
}

int dq8_decode_accumulate_avg_local(int kind, const uint8_t *const *codes, const float *const *scales, int K,
                                    const float *local, size_t n, size_t block, float *out, void *hip_stream)
{
    static const char who[] = "dq8_decode_accumulate_avg_local";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (K < 0 || K > DQ8_MAX_K) return fail(DQ8_ERR_ARG, "%s: K = %d outside 0..%d", who, K, DQ8_MAX_K);
    if (n == 0) return DQ8_OK;
    if (!local || !out) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "%s: n too large", who);
    const size_t Bq = (block == 0 || block > n) ? n : block;
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(out, n * 4, local, n * 4)) return fail(DQ8_ERR_ARG, "%s: out overlaps local", who);
    WorkerPtrs wp;
    rc = gather_workers(who, codes, scales, K, n, nbq, out, n * 4, &wp);
    if (rc) return rc;
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    if ((K == 2 || K == 4 || K == 8) && g_tune.avg_lean) {
        const Plan p = make_plan(n, block, st->cus, 1, 1);
        bool launched = false;
        rc = launch_avg_full(*st, kind, wp, K, local, n, p, out, static_cast<hipStream_t>(hip_stream), &launched);
        if (rc || launched) return rc;
    }
    return launch_avg_block(*st, kind, wp, K, local, n, block, out, nullptr, nullptr, static_cast<hipStream_t>(hip_stream));
}

int dq8_decode_avg_encode(int kind, const uint8_t *const *codes, const float *const *scales, int K, const float *local,
                          size_t n, size_t block, float *out_scales, uint8_t *out_codes, void *hip_stream)
{
    static const char who[] = "dq8_decode_avg_encode";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (K < (local ? 0 : 1) || K > DQ8_MAX_K)
        return fail(DQ8_ERR_ARG, "%s: K = %d outside %d..%d", who, K, local ? 0 : 1, DQ8_MAX_K);
    if (n == 0) return DQ8_OK;
    if (!out_scales || !out_codes) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "%s: n too large", who);
    const size_t Bq = (block == 0 || block > n) ? n : block;
    const size_t nbq = (n + Bq - 1) / Bq;
    if (Bq > (size_t)kUnit)
        return fail(DQ8_ERR_ARG, "%s: a scale block of %zu elements does not fit the registers of a wavefront (at most %d); "
                    "use dq8_decode_accumulate_avg and dq8_encode", who, Bq, kUnit);
    if (overlaps(out_codes, n, out_scales, nbq * 4)) return fail(DQ8_ERR_ARG, "%s: outputs overlap", who);
    if (local && (overlaps(out_codes, n, local, n * 4) || overlaps(out_scales, nbq * 4, local, n * 4)))
        return fail(DQ8_ERR_ARG, "%s: an output overlaps local", who);
    WorkerPtrs wp;
    rc = gather_workers(who, codes, scales, K, n, nbq, out_codes, n, &wp);
    if (rc) return rc;
    rc = gather_workers(who, codes, scales, K, n, nbq, out_scales, nbq * 4, &wp);
    if (rc) return rc;
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    return launch_avg_block(*st, kind, wp, K, local, n, block, nullptr, out_scales, out_codes,
                            static_cast<hipStream_t>(hip_stream));
}

int dq8_error_stats(int kind, const float *x, size_t n, size_t block, float *scales, unsigned flags, double *stats,
                    double *means, void *hip_stream)
{
    static const char who[] = "dq8_error_stats";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (flags & ~DQ8_SCALES_GIVEN) return fail(DQ8_ERR_ARG, "%s: unknown flags 0x%x", who, flags);
    if (n == 0) return DQ8_OK;
    if (!x || !scales || !stats) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "%s: n too large", who);
    if (((uintptr_t)stats & 7) || ((uintptr_t)means & 7)) return fail(DQ8_ERR_ARG, "%s: stats and means must be 8-byte aligned", who);
    const size_t Bq = (block == 0 || block > n) ? n : block;
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(stats, nbq * 32, x, n * 4) || overlaps(stats, nbq * 32, scales, nbq * 4) || overlaps(scales, nbq * 4, x, n * 4) ||
        (means && (overlaps(means, 16, x, n * 4) || overlaps(means, 16, scales, nbq * 4) || overlaps(means, 16, stats, nbq * 32))))
        return fail(DQ8_ERR_ARG, "%s: buffers overlap", who);
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!(flags & DQ8_SCALES_GIVEN)) {
        rc = launch_absmax(*st, x, n, block, scales, stream);
        if (rc) return rc;
    }
    return launch_error_stats(*st, kind, x, n, block, scales, stats, means, stream);
}

int dq8_model_penalty(const double *transfer_ms, const double *compute_ms, size_t count, double *penalty_ms)
{
    if (!penalty_ms || (count > 0 && (!transfer_ms || !compute_ms))) return fail(DQ8_ERR_NULL, "dq8_model_penalty: NULL pointer");
    double total = 0.0;
    for (size_t i = 0; i < count; ++i) {
        if (!(transfer_ms[i] >= 0.0) || !(compute_ms[i] >= 0.0) || transfer_ms[i] > 1e300 || compute_ms[i] > 1e300)
            return fail(DQ8_ERR_ARG, "dq8_model_penalty: entry %zu is negative or not finite", i);
        const double open_part = transfer_ms[i] - compute_ms[i];
        total = total + (open_part > 0.0 ? open_part : 0.0);
    }
    *penalty_ms = total;
    return DQ8_OK;
}

int dq8_model_speedup(int n_gpus, double total_ms, double fc_ms, double conv_penalty_ms, int sub_batches,
                      double parallel_fc_ms, double fc_penalty_ms, double *speedup)
{
    if (!speedup) return fail(DQ8_ERR_NULL, "dq8_model_speedup: speedup is NULL");
    const double t[5] = {total_ms, fc_ms, conv_penalty_ms, parallel_fc_ms, fc_penalty_ms};
    for (double v : t)
        if (!(v >= 0.0) || v > 1e300) return fail(DQ8_ERR_ARG, "dq8_model_speedup: a time is negative or not finite");
    if (n_gpus < 1 || sub_batches < 0) return fail(DQ8_ERR_ARG, "dq8_model_speedup: n_gpus = %d, sub_batches = %d", n_gpus, sub_batches);
    if (fc_ms > total_ms) return fail(DQ8_ERR_ARG, "dq8_model_speedup: the fully connected part is longer than the whole pass");
    const double denominator = (total_ms - fc_ms) + conv_penalty_ms + sub_batches * parallel_fc_ms + fc_penalty_ms;
    if (!(denominator > 0.0)) return fail(DQ8_ERR_ARG, "dq8_model_speedup: the parallel pass takes no time");
    *speedup = n_gpus * total_ms / denominator;
    return DQ8_OK;
}

// ---- internal entry points used by the CPU tests of the host logic (dq8_internal.h)

int dq8_internal_tables(int kind, float *cb256, float *thr127, uint32_t *lo_key, uint32_t *n_bucket, uint32_t *bucket,
                        uint32_t bucket_capacity)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    if (cb256) std::memcpy(cb256, t.cb, sizeof(t.cb));
    if (thr127) std::memcpy(thr127, t.thr, sizeof(t.thr));
    if (lo_key) *lo_key = t.lo_key;
    if (n_bucket) *n_bucket = t.n_bucket;
    if (bucket) {
        if (bucket_capacity < t.n_bucket) return fail(DQ8_ERR_ARG, "bucket buffer too small");
        std::memcpy(bucket, t.bucket, sizeof(uint32_t) * t.n_bucket);
    }
    return DQ8_OK;
}

int dq8_internal_ranks(int kind, uint32_t *n_mag, uint8_t *canon128)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    if (n_mag) *n_mag = t.n_mag;
    if (canon128) std::memcpy(canon128, t.canon, sizeof(t.canon));
    return DQ8_OK;
}

int dq8_internal_plan(size_t n, size_t block, int cus, int waves_per_cu, int wpb, size_t unit, size_t *out6)
{
    if (!out6 || cus < 1 || waves_per_cu < 1 || (wpb != 1 && wpb != 4) || unit < 256 || (unit & (unit - 1)))
        return fail(DQ8_ERR_ARG, "dq8_internal_plan: bad argument");
    Plan p = make_plan(n, block, cus, waves_per_cu, wpb, kWavesPerWg, unit);
    out6[0] = p.B;
    out6[1] = p.nb;
    out6[2] = p.upb;
    out6[3] = p.n_units;
    out6[4] = p.n_teams;
    out6[5] = p.grid;
    return DQ8_OK;
}

int dq8_internal_tune(const char *key, int value)
{
    if (!key) return fail(DQ8_ERR_NULL, "dq8_internal_tune: key is NULL");
    struct { const char *name; int *slot; int lo, hi; } keys[] = {
        {"amax_nt", &g_tune.amax_nt, 0, 1}, 
        {"avg_lean", &g_tune.avg_lean, 0, 1}, {"avg_lean_q", &g_tune.avg_lean_q, 2, 4},
        {"avg_lean_wpc", &g_tune.avg_lean_wpc, 1, 32}, {"avg_lean_wpw", &g_tune.avg_lean_wpw, 4, 16}, {"copy_nt", &g_tune.copy_nt, 0, 2},           {"fastdiv", &g_tune.fastdiv, 0, 1},   {"enc_wpb", &g_tune.enc_wpb, 1, 4},
        {"enc_wpc", &g_tune.enc_wpc, 1, 32}, {"enc_lean", &g_tune.enc_lean, 0, 1}, {"enc_lean_wpc", &g_tune.enc_lean_wpc, 4, 32}, {"enc_fill", &g_tune.enc_fill, 0, 1}, {"amax_q", &g_tune.amax_q, 1, 16},    {"amax_wpc", &g_tune.amax_wpc, 1, 32},
        {"dec_q", &g_tune.dec_q, 1, 16},     {"dec_wpc", &g_tune.dec_wpc, 1, 32},  {"avg_q", &g_tune.avg_q, 1, 4},
        {"avg_wpc", &g_tune.avg_wpc, 1, 32}, {"avg_wpw", &g_tune.avg_wpw, 4, 16}, {"dec_wpw", &g_tune.dec_wpw, 4, 16}, {"blk_wpw", &g_tune.blk_wpw, 6, 8}, {"avg_team", &g_tune.avg_team, 0, 1}, {"avg_steady", &g_tune.avg_steady, 0, 1}, {"avg_teams", &g_tune.avg_teams, 2, 4}, {"avg_wgpc", &g_tune.avg_wgpc, 1, 2}, {"copy_q", &g_tune.copy_q, 1, 16},    {"copy_wpc", &g_tune.copy_wpc, 1, 32},
    };
    for (auto &k : keys)
        if (!std::strcmp(k.name, key)) {
            if (value < k.lo || value > k.hi) return fail(DQ8_ERR_ARG, "dq8_internal_tune: %s = %d outside %d..%d", key, value, k.lo, k.hi);
            *k.slot = value;
            return DQ8_OK;
        }
    return fail(DQ8_ERR_ARG, "dq8_internal_tune: unknown key %s", key);
}

int dq8_internal_copy(float *dst, const float *src, size_t n, void *hip_stream)
{
    if (n == 0) return DQ8_OK;
    if (!dst || !src) return fail(DQ8_ERR_NULL, "dq8_internal_copy: NULL pointer");
    DeviceState *st;
    int rc = device_state(&st);
    if (rc) return rc;
    const int q = (g_tune.copy_q == 1 || g_tune.copy_q == 2 || g_tune.copy_q == 8 || g_tune.copy_q == 16) ? g_tune.copy_q : 4;
    Plan p = make_plan(n, 0, st->cus, g_tune.copy_wpc, 1, kWavesPerWg, (size_t)q * 4 * kWave);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
#define DQ8_COPY(Q, NT) \
    hipLaunchKernelGGL((k_copy<Q, NT>), dim3(p.grid), dim3(kWg), 0, stream, src, dst, n, p.n_units, p.n_teams)
#define DQ8_COPY_Q(NT)                   \
    switch (q) {                         \
    case 1: DQ8_COPY(1, NT); break;      \
    case 2: DQ8_COPY(2, NT); break;      \
    case 8: DQ8_COPY(8, NT); break;      \
    case 16: DQ8_COPY(16, NT); break;    \
    default: DQ8_COPY(4, NT); break;     \
    }
    switch (g_tune.copy_nt) {
    case 0: DQ8_COPY_Q(0) break;
    case 2: DQ8_COPY_Q(2) break;
    default: DQ8_COPY_Q(1) break;
    }
#undef DQ8_COPY_Q
#undef DQ8_COPY
    return after_launch("k_copy");
}

static int host_search(int kind, Search *sr)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    static thread_local uint32_t remap[kRemapWords];
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    for (int r = 0; r < kRemapWords; ++r) remap[r] = t.canon[r];
    *sr = make_search(t.bucket, t.lo_key, t.n_bucket, t.has_remap ? remap : nullptr);
    return DQ8_OK;
}

int dq8_internal_check_search(int kind, uint64_t *mismatches, uint64_t *missed_near)
{
    Search sr;
    int rc = host_search(kind, &sr);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    dq8::build_tables(kind, &t);
    const uint32_t n_thr = t.n_mag - 1;
    uint32_t thr_bits[127];
    std::memcpy(thr_bits, t.thr, sizeof(thr_bits));
    uint64_t bad = 0, missed = 0;
    uint32_t j = 0;  // thresholds <= the current value = rank of the nearest magnitude
    for (uint32_t bits = 0; bits <= 0x7F800000u; ++bits) {
        while (j < n_thr && thr_bits[j] <= bits) ++j;
        const float pos = u2f(bits), neg = u2f(bits | 0x80000000u);
        const uint32_t sp = search_sum(sr, pos), sn = search_sum(sr, neg);
        const uint32_t want = t.canon[j];
        bad += code_of(sr, sp, pos) != want;
        bad += code_of(sr, sn, neg) != (want | 0x80u);
        // every value within kNearWindow steps of a threshold must raise the proximity flag
        bool close = (j < n_thr && thr_bits[j] - bits <= kNearWindow) || (j > 0 && bits - thr_bits[j - 1] <= kNearWindow);
        if (close && near_key(sp) > 2 * kNearWindow) ++missed;
    }
    if (mismatches) *mismatches = bad;
    if (missed_near) *missed_near = missed;
    return DQ8_OK;
}

int dq8_internal_encode_host(int kind, const float *x, size_t n, float scale, int use_reciprocal, uint8_t *codes,
                             uint64_t *n_exact)
{
    Search sr;
    int rc = host_search(kind, &sr);
    if (rc) return rc;
    const float d = scale == 0.0f ? 1.0f : scale;
    const float r = 1.0f / d;
    const bool recip = use_reciprocal && reciprocal_ok(d);
    uint64_t exact = 0;
    for (size_t i = 0; i < n; ++i) {
        if (recip) {
            uint32_t s0 = search_sum(sr, x[i] * r);
            if (near_key(s0) > 2 * kNearWindow) {
                codes[i] = (uint8_t)code_of(sr, s0, x[i]);
                continue;
            }
        }
        ++exact;
        codes[i] = (uint8_t)code_exact(sr, x[i], d);
    }
    if (n_exact) *n_exact = exact;
    return DQ8_OK;
}

}  // extern "C"
