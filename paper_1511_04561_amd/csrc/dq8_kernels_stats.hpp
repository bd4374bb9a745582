// dq8 kernels for the approximation-error statistics.
#pragma once
#include "dq8_device.hpp"

namespace {

// Approximation-error statistics of compress-then-decompress (Sec. 3.4, Table 2).  Per block b,
// stats[4 b + 0] = sum of e, [1] = sum of e / |x| over x != 0, [2] = number of x != 0,
// [3] = largest e, with q = fl32(cb[code] * s) and e = |(double) q - (double) x| (one binary64
// subtraction; the quotient one correctly rounded binary64 division).
//
// What a lane does per element.  The code's sign is the sign of x (scales are not negative), so q and x have
// the same sign and e = | |q| - |x| |: the kernel works on magnitudes and never forms the code byte.  |q| comes
// from a table in LDS that is indexed by byte 2 of the search sum (the code field, marked or not, see
// fix_marked_codes) and holds one copy per lane, so the lookup address is one byte permute and no two lanes
// meet in a bank.  The number of non-zero inputs is counted on the scalar unit from the lanes' votes.
//
// The quotient e / |x|.  Both operands are binary32 magnitudes widened to binary64 (e is a difference of two of
// them): 0 <= e < 2^129, 2^-149 <= |x| < 2^128.  The quotient and every intermediate of the division are
// therefore normal binary64 numbers far from overflow and underflow, which is the one case in which the
// division's range reduction, its rescaling and its special-case selection do nothing.  What is left is the
// reciprocal estimate, two Newton steps on it, the quotient estimate and its correction with the exactly
// computed remainder, which yields the correctly rounded quotient (same operations, same order as the general
// division).
__device__ __forceinline__ double quotient_of_magnitudes(double e, double ax)
{
    double r = __builtin_amdgcn_rcp(ax);
    r = __builtin_fma(__builtin_fma(-ax, r, 1.0), r, r);
    r = __builtin_fma(__builtin_fma(-ax, r, 1.0), r, r);
    const double q = e * r;
    return __builtin_fma(__builtin_fma(-ax, q, e), r, q);
}

// Magnitude table for the lookup above: row b (b = 0 .. 255, a possibly marked code byte) holds the table value
// of the code that byte stands for, 64 copies (one per lane); entry (b, lane) at byte address b * 256 + lane * 4.
// Thread t < 256 fills row t.  The caller synchronises before the first lookup.
__device__ __forceinline__ void load_magnitude_lut(const uint32_t *tab, float *lds)
{
    if (threadIdx.x < 256) {
        const uint32_t code = fix_marked_codes(threadIdx.x) & 0x7Fu;
        const float val = u2f(tab[kCbOff + code]);
        const v4f four = {val, val, val, val};
        v4f *row = reinterpret_cast<v4f *>(lds + threadIdx.x * kLutCopies);
#pragma unroll
        for (int c = 0; c < kLutCopies / 4; ++c) row[c] = four;
    }
}

// wavefronts per workgroup: two workgroups (two value tables) share a compute unit, six wavefronts per SIMD
// (88.4 us with 8, 85.4 us with 12, 106 us with 16, where the registers no longer suffice)
constexpr int kStatsWaves = 12;
constexpr int kStatsWg = kStatsWaves * kWave;

// Running statistics of one wavefront for the block it is in.
struct ErrorSums {
    double sum_abs = 0.0, sum_rel = 0.0, worst = 0.0;
    uint64_t count = 0;  // wave-uniform: non-zero inputs of all lanes so far
};

// OWN = true: a wavefront owns whole blocks (block b of round i goes to wavefront b - i * n_waves; the blocks of the
// last, partial round are spread evenly over the wavefronts), adds a block's terms in a fixed order and stores the
// four numbers: no atomics, stats[] need not be zeroed, and the sums are the same in every launch.
// OWN = false (blocks too long or too few for that): a wavefront walks a contiguous run of `per_wave` units and
// merges its sums into stats[], which the host has zeroed, with atomics when the block changes and at the end:
// the count and the maximum are exact in any order (integers below 2^53, and non-negative binary64 numbers order
// like their bit patterns); the two sums depend on the order only in their last bits.
// Units are Q * 256 elements; the loads of a wavefront's next unit are issued before the current one is worked on.
template <int Q, bool OWN>
__global__ __launch_bounds__(kStatsWg, kStatsWaves / 2) void k_error_stats(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                         size_t n, size_t B, size_t nb, size_t upb, size_t n_units,
                                                         size_t per_wave, size_t n_waves,
                                                         const float *__restrict__ scales, double *__restrict__ stats)
{
    constexpr int U = Q * 4 * kWave;
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t bucket_lds[];
    load_magnitude_lut(tab, lut);
    const Search sr = load_bucket_table(tab, bucket_lds, kStatsWg);
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    const size_t wave = first_unit(kStatsWaves);

    ErrorSums acc;
    auto add = [&](float xv, float qmag) {
        const double ax = (double)__builtin_fabsf(xv);
        const double e = __builtin_fabs((double)qmag - ax);
        acc.sum_abs += e;
        acc.worst = __builtin_fmax(acc.worst, e);
        const bool nz = xv != 0.0f;
        acc.count += (uint64_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(nz));
        // no branch around the division: a zero's quotient is computed (it is a NaN) and not added, so that the
        // elements of a unit stay in one stretch of code that the scheduler can interleave
        const double rel = quotient_of_magnitudes(e, ax);
        acc.sum_rel += nz ? rel : 0.0;
    };
    // The wave's sums for block blk: a fixed tree over the lanes, then lane 0 stores or merges them.
    auto flush = [&](size_t blk) {
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            acc.sum_abs += __shfl_xor(acc.sum_abs, m);
            acc.sum_rel += __shfl_xor(acc.sum_rel, m);
            acc.worst = __builtin_fmax(acc.worst, __shfl_xor(acc.worst, m));
        }
        if (lane == 0) {
            double *p = stats + 4 * blk;
            if (OWN) {
                p[0] = acc.sum_abs;
                p[1] = acc.sum_rel;
                p[2] = (double)acc.count;
                p[3] = acc.worst;
            } else {
                atomicAdd(p, acc.sum_abs);
                atomicAdd(p + 1, acc.sum_rel);
                atomicAdd(p + 2, (double)acc.count);
                atomicMax(reinterpret_cast<unsigned long long *>(p + 3), (unsigned long long)__double_as_longlong(acc.worst));
            }
        }
        acc = ErrorSums();
    };
    // One unit whose quads are in v (whole, aligned) or that is read element by element.
    auto work = [&](const Unit &un, bool fast, const v4f (&v)[Q]) {
        const float s = scales[un.block];
        const float sa = __builtin_fabsf(s);
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        if (fast) {
            uint32_t sum[Q][4];
            if (recip) {
                uint32_t all = 0xFFFFu;
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    sum[j][0] = search_sum(sr, v[j].x * r);
                    sum[j][1] = search_sum(sr, v[j].y * r);
                    sum[j][2] = search_sum(sr, v[j].z * r);
                    sum[j][3] = search_sum(sr, v[j].w * r);
                }
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const uint32_t k01 = near_key(sum[j][0]) < near_key(sum[j][1]) ? near_key(sum[j][0]) : near_key(sum[j][1]);
                    const uint32_t k23 = near_key(sum[j][2]) < near_key(sum[j][3]) ? near_key(sum[j][2]) : near_key(sum[j][3]);
                    const uint32_t k = k01 < k23 ? k01 : k23;
                    all = all < k ? all : k;
                }
                // some value of some lane lies next to a threshold: the whole unit again with true divisions
                if (__builtin_amdgcn_ballot_w64(all <= 2 * kNearWindow) != 0) {
#pragma unroll
                    for (int j = 0; j < Q; ++j) {
                        sum[j][0] = search_sum_exact(sr, v[j].x / d);
                        sum[j][1] = search_sum_exact(sr, v[j].y / d);
                        sum[j][2] = search_sum_exact(sr, v[j].z / d);
                        sum[j][3] = search_sum_exact(sr, v[j].w / d);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    sum[j][0] = search_sum_exact(sr, v[j].x / d);
                    sum[j][1] = search_sum_exact(sr, v[j].y / d);
                    sum[j][2] = search_sum_exact(sr, v[j].z / d);
                    sum[j][3] = search_sum_exact(sr, v[j].w / d);
                }
            }
            // byte 1 of the address = byte 2 of the sum (the code field), byte 0 = lane * 4
            auto magnitude = [&](uint32_t sm) {
                const uint32_t addr = __builtin_amdgcn_perm(sm, lane4, 0x0C0C0600u);
                return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lut) + addr) * sa;
            };
            float qm[Q][4];  // all lookups first, so that their latencies overlap
#pragma unroll
            for (int j = 0; j < Q; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c) qm[j][c] = magnitude(sum[j][c]);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                add(v[j].x, qm[j][0]);
                add(v[j].y, qm[j][1]);
                add(v[j].z, qm[j][2]);
                add(v[j].w, qm[j][3]);
            }
        } else {
            const float *px = x + un.start;
            for (uint32_t i0 = 0; i0 < un.len; i0 += kWave) {  // every lane takes part in the votes of add()
                const uint32_t i = i0 + lane;
                const bool in = i < un.len;
                const float xv = in ? px[i] : 0.0f;
                const uint32_t sm = search_sum_exact(sr, xv / d);
                const uint32_t addr = __builtin_amdgcn_perm(sm, lane4, 0x0C0C0600u);
                const float q = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lut) + addr) * sa;
                add(xv, in ? q : 0.0f);  // a lane past the end adds e = 0 and no count
            }
        }
    };
    auto is_fast = [&](const Unit &un) { return un.len == (uint32_t)U && (((uintptr_t)(x + un.start)) & 15) == 0; };
    auto load = [&](const Unit &un, v4f (&v)[Q]) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x + un.start);
#pragma unroll
        for (int j = 0; j < Q; ++j) v[j] = ldg<1>(p4 + j * kWave + lane);
    };

    if (OWN) {
        // blocks of this wavefront: one per full round, and possibly one of the last round
        const size_t rounds = nb / n_waves, rem = nb - rounds * n_waves;
        const size_t extra_lo = wave * rem / n_waves, extra_hi = (wave + 1) * rem / n_waves;
        const size_t mine = rounds + (extra_hi > extra_lo ? 1 : 0);
        if (mine == 0) return;
        auto block_of = [&](size_t i) { return i < rounds ? i * n_waves + wave : rounds * n_waves + extra_lo; };
        v4f va[Q], vb[Q];
        size_t i = 0, c = 0;  // block number i of this wavefront, unit c of it
        Unit cur = unit_of<U>(block_of(0) * upb, n, B, nb, upb);
        bool cur_fast = is_fast(cur);
        if (cur_fast) load(cur, va);
        for (;;) {
            // the unit after this one: the next of the block, or the first of the wavefront's next block
            size_t ni = i, nc = c + 1;
            if (nc * (size_t)U >= (size_t)(B < n - cur.block * B ? B : n - cur.block * B)) {
                ni = i + 1;
                nc = 0;
            }
            const bool more = ni < mine;
            Unit nxt = cur;
            bool nxt_fast = false;
            if (more) {
                nxt = unit_of<U>(block_of(ni) * upb + nc, n, B, nb, upb);
                nxt_fast = is_fast(nxt);
                if (nxt_fast) load(nxt, vb);
            }
            work(cur, cur_fast, va);
            if (!more || ni != i) flush(cur.block);
            if (!more) break;
            for (int j = 0; j < Q; ++j) va[j] = vb[j];
            cur = nxt;
            cur_fast = nxt_fast;
            i = ni;
            c = nc;
        }
    } else {
        const size_t u0 = wave * per_wave;
        const size_t u1 = u0 + per_wave < n_units ? u0 + per_wave : n_units;
        if (u0 >= u1) return;
        v4f va[Q], vb[Q];
        Unit cur = unit_of<U>(u0, n, B, nb, upb);
        bool cur_fast = is_fast(cur);
        if (cur_fast) load(cur, va);
        for (size_t u = u0; u < u1; ++u) {
            const bool more = u + 1 < u1;
            Unit nxt = cur;
            bool nxt_fast = false;
            if (more) {
                nxt = unit_of<U>(u + 1, n, B, nb, upb);
                nxt_fast = is_fast(nxt);
                if (nxt_fast) load(nxt, vb);
            }
            work(cur, cur_fast, va);
            if (!more || nxt.block != cur.block) flush(cur.block);
            for (int j = 0; j < Q; ++j) va[j] = vb[j];
            cur = nxt;
            cur_fast = nxt_fast;
        }
    }
}

// Means over all blocks from the per-block statistics: means[0] = (sum of absolute errors) / n,
// means[1] = (sum of relative errors) / (number of non-zero inputs), 0 when there is none.
// One workgroup of 1024 threads; thread t adds blocks t, t + 1024, ... in that order and the threads'
// sums are combined by a fixed tree, so the result is the same in every launch.  (A separate launch because a
// fold into the statistics kernel would need a grid-wide counter, and the library keeps no device memory of
// its own that concurrent calls could share.)
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

}  // namespace
