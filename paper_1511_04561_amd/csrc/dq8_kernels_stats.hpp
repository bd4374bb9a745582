// dq8 kernels for the approximation-error statistics.
#pragma once
#include "dq8_device.hpp"

namespace {

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

}  // namespace
