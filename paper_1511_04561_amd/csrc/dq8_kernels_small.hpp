// dq8 kernels for short scale blocks: 4, 8, 16, 32, 64 or 128 elements per block (up to 1024 where a block has
// to be held: compression and average-then-compress; a block is then one, two or four whole rows of a unit).
//
// The other kernels give a wavefront one piece of one block at a time, which leaves most lanes idle
// when a block has fewer than 256 elements.  Here a wavefront takes units of Q * 256 elements that
// hold many whole blocks: lane L owns quad j * 64 + L of the unit (j = 0 .. Q - 1), a block is
// G = block / 4 neighbouring lanes of one such row, the block maximum is a reduction over those G
// lanes (data-parallel-primitive steps, no LDS), and every lane works with its own block's scale.
// The arithmetic per element is that of the other kernels, so the results are identical.
// The host launches these for whole units only (16-byte aligned fp32 arrays, 4-byte aligned codes) and
// hands the remaining elements, a whole number of blocks from a block boundary on, to the general kernels.
#pragma once
#include "dq8_device.hpp"

namespace {

// Maximum over each group of G neighbouring lanes (G a power of two up to 64), in every lane of the group.
template <int G>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v)
{
    static_assert(G >= 1 && G <= 64 && (G & (G - 1)) == 0, "groups are powers of two inside a wavefront");
    if (G == 64) return wave_max_u32(v);
    if (G >= 2) v = max_dpp<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
    if (G >= 4) v = max_dpp<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
    if (G >= 8) v = max_dpp<0x141, 0xF>(v);  // row_half_mirror
    if (G >= 16) v = max_dpp<0x140, 0xF>(v); // row_mirror
    if (G >= 32) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, 16);
        v = o > v ? o : v;
    }
    return v;
}

// Four codes of one quad when every lane has its own divisor d (positive).  The reciprocal path is taken
// when no lane of the wavefront objects: a lane objects when its product lies next to a threshold or a bucket
// edge, or when its divisor is outside the range in which the product is within three steps of the quotient.
__device__ __forceinline__ uint32_t encode_quad_own_scale(const Search &sr, v4f v, float d)
{
    const float r = 1.0f / d;
    const uint32_t s0 = search_sum(sr, v.x * r), s1 = search_sum(sr, v.y * r);
    const uint32_t s2 = search_sum(sr, v.z * r), s3 = search_sum(sr, v.w * r);
    uint32_t k0 = near_key(s0), k1 = near_key(s1), k2 = near_key(s2), k3 = near_key(s3);
    k0 = k0 < k1 ? k0 : k1;
    k2 = k2 < k3 ? k2 : k3;
    k0 = k0 < k2 ? k0 : k2;
    if (!reciprocal_ok(d)) k0 = 0;
    if (__builtin_amdgcn_ballot_w64(k0 <= 2 * kNearWindow) == 0) return pack_codes(sr, s0, s1, s2, s3, v);
    return pack_codes(sr, search_sum_exact(sr, v.x / d), search_sum_exact(sr, v.y / d), search_sum_exact(sr, v.z / d), search_sum_exact(sr, v.w / d), v);
}

// Index of the block that holds this lane's quad j of unit u.
template <int Q, int G>
__device__ __forceinline__ size_t small_block_of(size_t u, int j, uint32_t lane)
{
    constexpr int kBlocksPerUnit = Q * kWave / G;
    return u * (size_t)kBlocksPerUnit + (uint32_t)(j * kWave + lane) / (uint32_t)G;
}

// Block maxima of whole units.
template <int Q, int G>
__global__ __launch_bounds__(kWg) void k_small_absmax(const float *__restrict__ x, size_t n_units, size_t n_waves,
                                                     float *__restrict__ scales)
{
    constexpr int U = Q * 4 * kWave;
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x) + u * (U / 4);
        v4f v[Q];
#pragma unroll
        for (int j = 0; j < Q; ++j) v[j] = ldg_at<1>(p4, j * kWave + lane);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint32_t m = group_max_u32<G>(f2u(max4_abs(v[j], 0.0f)));
            if (lane % G == 0) scales[small_block_of<Q, G>(u, j, lane)] = u2f(m);
        }
    }
}

// Compression of whole units; GIVEN: the scales are read, otherwise computed as above and stored.
template <int Q, int G, bool GIVEN>
__global__ __launch_bounds__(kWg) void k_small_encode(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                     size_t n_units, size_t n_waves, float *__restrict__ scales,
                                                     uint8_t *__restrict__ codes)
{
    constexpr int U = Q * 4 * kWave;
    constexpr int R = G > kWave ? G / kWave : 1;  // rows of 64 quads per block
    constexpr int GL = G > kWave ? kWave : G;     // lanes of a row that belong to one block
    static_assert(Q % R == 0, "a block does not straddle units");
    extern __shared__ uint32_t lds[];
    const Search sr = load_bucket_table(tab, lds);
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x) + u * (U / 4);
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes) + u * (U / 4);
        v4f v[Q];
#pragma unroll
        for (int j = 0; j < Q; ++j) v[j] = ldg_at<1>(p4, j * kWave + lane);
#pragma unroll
        for (int j0 = 0; j0 < Q; j0 += R) {  // R rows of the unit share a block when a block is longer than a row
            const size_t blk = small_block_of<Q, G>(u, j0, lane);
            float s;
            if (GIVEN) {
                s = scales[blk];
            } else {
                float fm = 0.0f;
#pragma unroll
                for (int r = 0; r < R; ++r) fm = max4_abs(v[j0 + r], fm);
                s = u2f(group_max_u32<GL>(f2u(fm)));
                if (lane % GL == 0) scales[blk] = s;
            }
            const float d = s == 0.0f ? 1.0f : s;  // a zero scale leaves the value as it is
#pragma unroll
            for (int r = 0; r < R; ++r) stg_at<1>(c4, (j0 + r) * kWave + lane, encode_quad_own_scale(sr, v[j0 + r], d));
        }
    }
}

// Decompression of whole units.
template <int Q, int G, int WPW>
__global__ __launch_bounds__(kWave * WPW) void k_small_decode(const uint32_t *__restrict__ tab, const uint8_t *__restrict__ codes,
                                                             const float *__restrict__ scales, size_t n_units,
                                                             size_t n_waves, float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    load_lut(tab, lut);
    __syncthreads();
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    for (size_t u = first_unit(WPW); u < n_units; u += n_waves) {
        const uint32_t *c4 = reinterpret_cast<const uint32_t *>(codes) + u * (U / 4);
        v4f *o4 = reinterpret_cast<v4f *>(out) + u * (U / 4);
        uint32_t w[Q];
        float s[Q];
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            w[j] = ldg_at<1>(c4, j * kWave + lane);
            s[j] = scales[small_block_of<Q, G>(u, j, lane)];
        }
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            v4f r;
            r.x = lut_at<0>(lut, w[j], lane4) * s[j];
            r.y = lut_at<1>(lut, w[j], lane4) * s[j];
            r.z = lut_at<2>(lut, w[j], lane4) * s[j];
            r.w = lut_at<3>(lut, w[j], lane4) * s[j];
            stg<2>(o4 + j * kWave + lane, r);
        }
    }
}

// K-way decode-and-average of whole units, any K; `local` (may be NULL) is the first term.
template <int Q, int G, int WPW>
__global__ __launch_bounds__(kWave * WPW) void k_small_avg(const uint32_t *__restrict__ tab, WorkerPtrs p, int K,
                                                          const float *__restrict__ local, size_t n_units, size_t n_waves,
                                                          float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    load_lut(tab, lut);
    __syncthreads();
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    for (size_t u = first_unit(WPW); u < n_units; u += n_waves) {
        v4f *o4 = reinterpret_cast<v4f *>(out) + u * (U / 4);
        v4f acc[Q];
        if (local) {
            const v4f *l4 = reinterpret_cast<const v4f *>(local) + u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) {  // the sum starts at +0: a local -0 becomes +0
                const v4f l = ldg_at<1>(l4, j * kWave + lane);
                acc[j] = v4f{0.0f + l.x, 0.0f + l.y, 0.0f + l.z, 0.0f + l.w};
            }
        } else {
#pragma unroll
            for (int j = 0; j < Q; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        }
        for (int k = 0; k < K; ++k) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k]) + u * (U / 4);
            uint32_t w[Q];
            float s[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                w[j] = ldg_at<1>(c4, j * kWave + lane);
                s[j] = p.scales[k][small_block_of<Q, G>(u, j, lane)];
            }
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                acc[j].x = acc[j].x + lut_at<0>(lut, w[j], lane4) * s[j];
                acc[j].y = acc[j].y + lut_at<1>(lut, w[j], lane4) * s[j];
                acc[j].z = acc[j].z + lut_at<2>(lut, w[j], lane4) * s[j];
                acc[j].w = acc[j].w + lut_at<3>(lut, w[j], lane4) * s[j];
            }
        }
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            acc[j].x = mean_of(acc[j].x);
            acc[j].y = mean_of(acc[j].y);
            acc[j].z = mean_of(acc[j].z);
            acc[j].w = mean_of(acc[j].w);
            stg<2>(o4 + j * kWave + lane, acc[j]);
        }
    }
}

// Average-then-compress of whole units: the means of k_small_avg, each block's maximum over its lanes, and the
// compression of the means from the registers.  `local` (may be NULL) is the first term of the sum.
template <int Q, int G, int WPW>
__global__ __launch_bounds__(kWave * WPW) void k_small_avg_encode(const uint32_t *__restrict__ tab, WorkerPtrs p, int K,
                                                                 const float *__restrict__ local, size_t n_units,
                                                                 size_t n_waves, float *__restrict__ scales_out,
                                                                 uint8_t *__restrict__ codes_out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t bucket_lds[];
    constexpr int U = Q * 4 * kWave;
    constexpr int R = G > kWave ? G / kWave : 1;  // rows of 64 quads per block
    constexpr int GL = G > kWave ? kWave : G;     // lanes of a row that belong to one block
    static_assert(Q % R == 0, "a block does not straddle units");
    load_lut(tab, lut);
    const Search sr = load_bucket_table(tab, bucket_lds, kWave * WPW);
    __syncthreads();
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    for (size_t u = first_unit(WPW); u < n_units; u += n_waves) {
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out) + u * (U / 4);
        v4f acc[Q];
        if (local) {
            const v4f *l4 = reinterpret_cast<const v4f *>(local) + u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) {  // the sum starts at +0: a local -0 becomes +0
                const v4f l = ldg_at<1>(l4, j * kWave + lane);
                acc[j] = v4f{0.0f + l.x, 0.0f + l.y, 0.0f + l.z, 0.0f + l.w};
            }
        } else {
#pragma unroll
            for (int j = 0; j < Q; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        }
        for (int k = 0; k < K; ++k) {
            const uint32_t *w4 = reinterpret_cast<const uint32_t *>(p.codes[k]) + u * (U / 4);
            uint32_t w[Q];
            float s[Q];
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                w[j] = ldg_at<1>(w4, j * kWave + lane);
                s[j] = p.scales[k][small_block_of<Q, G>(u, j, lane)];
            }
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                acc[j].x = acc[j].x + lut_at<0>(lut, w[j], lane4) * s[j];
                acc[j].y = acc[j].y + lut_at<1>(lut, w[j], lane4) * s[j];
                acc[j].z = acc[j].z + lut_at<2>(lut, w[j], lane4) * s[j];
                acc[j].w = acc[j].w + lut_at<3>(lut, w[j], lane4) * s[j];
            }
        }
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            acc[j].x = mean_of(acc[j].x);
            acc[j].y = mean_of(acc[j].y);
            acc[j].z = mean_of(acc[j].z);
            acc[j].w = mean_of(acc[j].w);
        }
#pragma unroll
        for (int j0 = 0; j0 < Q; j0 += R) {  // R rows of the unit share a block when a block is longer than a row
            float fm = 0.0f;
#pragma unroll
            for (int r = 0; r < R; ++r) fm = max4_abs(acc[j0 + r], fm);
            const float s = u2f(group_max_u32<GL>(f2u(fm)));
            if (lane % GL == 0) scales_out[small_block_of<Q, G>(u, j0, lane)] = s;
            const float d = s == 0.0f ? 1.0f : s;
#pragma unroll
            for (int r = 0; r < R; ++r) stg_at<1>(c4, (j0 + r) * kWave + lane, encode_quad_own_scale(sr, acc[j0 + r], d));
        }
    }
}

}  // namespace
