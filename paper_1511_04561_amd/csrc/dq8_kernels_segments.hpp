// dq8 kernels for an array cut into segments of any lengths (tensors laid out back to back), one scale per
// segment: the paper's per-matrix maximum (Sec. 3.1, last paragraph) for a whole set of matrices in one launch
// instead of one call per matrix.
//
// bounds[0 .. n_seg] are element offsets, bounds[i] <= bounds[i + 1], segment i = [bounds[i], bounds[i + 1]).
// A workgroup copies them to LDS, every entry clamped to n, so that nothing the array holds can lead an access
// outside [0, n): the kernels walk the array in units of 1024 elements by position, and the segment of an
// element is looked up, never the elements of a segment.  Entries that do not ascend give meaningless
// results inside the arrays.
// A wavefront takes a unit at a time.  The segment of the unit's first element comes from two votes over
// the bounds (64 evenly spaced ones, then the 64 of the stretch the first vote names).  A unit that lies inside
// one segment and is a whole aligned unit takes the register path of the other kernels with that segment's
// scale; any other unit (a segment ends inside it, the end of the array, misaligned arrays) gives every lane
// sixteen consecutive elements: one binary search for the first, then a step to the next segment whenever an
// element reaches the next bound.
#pragma once
#include "dq8_device.hpp"

namespace {

constexpr int kSegMax = DQ8_MAX_SEGMENTS;           // segments per call: the bounds fit 32 KiB of LDS
constexpr int kSegRun = kSegUnit / kWave;           // 16 consecutive elements per lane on the slow path

// Copies bounds[0 .. n_seg] to LDS, clamped to n.  The caller synchronises the workgroup.
__device__ __forceinline__ void load_bounds(const uint64_t *__restrict__ bounds, uint32_t n_seg, size_t n, uint64_t *lds)
{
    for (uint32_t i = threadIdx.x; i <= n_seg; i += blockDim.x) {
        const uint64_t b = bounds[i];
        lds[i] = b < (uint64_t)n ? b : (uint64_t)n;
    }
}

// The last segment whose first element is at or before element v (the same v in every lane), at most
// n_seg - 1: two votes of the wavefront.
__device__ __forceinline__ uint32_t segment_of_uniform(const uint64_t *lds, uint32_t n_seg, uint64_t v, uint32_t lane)
{
    const uint32_t stride = (n_seg + kWave) / kWave;  // ceil((n_seg + 1) / 64), at most 64
    uint32_t i = lane * stride;
    i = i < n_seg ? i : n_seg;
    const uint32_t c1 = (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(lds[i] <= v && lane * stride <= n_seg));
    const uint32_t base = (c1 ? c1 - 1 : 0) * stride;
    uint32_t j = base + lane;
    const bool in = lane < stride && j <= n_seg;
    j = j < n_seg ? j : n_seg;
    const uint32_t c2 = (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(in && lds[j] <= v));
    const uint32_t s = base + (c2 ? c2 - 1 : 0);
    return s < n_seg - 1 ? s : n_seg - 1;
}

// The same for a v of the lane's own: binary search.
__device__ __forceinline__ uint32_t segment_of_lane(const uint64_t *lds, uint32_t n_seg, uint64_t v)
{
    uint32_t lo = 0, hi = n_seg;  // the answer is in [lo, hi)
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (lds[mid] <= v)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// Geometry of unit u and what it needs: its first element, its length, the segment of its first element and
// whether that segment holds the whole unit.
struct SegUnit {
    size_t start;
    uint32_t len, seg;
    bool single;
};

__device__ __forceinline__ SegUnit open_segment_unit(const uint64_t *lds, uint32_t n_seg, size_t n, size_t u, uint32_t lane)
{
    SegUnit q;
    q.start = u * (size_t)kSegUnit;
    q.len = cap_to_unit<kSegUnit>(n - q.start);
    q.seg = segment_of_uniform(lds, n_seg, q.start, lane);
    // (the last segment takes whatever lies beyond its end: bounds[n_seg] is n for well-formed bounds)
    q.single = q.seg == n_seg - 1 || lds[q.seg + 1] >= q.start + q.len;
    return q;
}

// Slow path: calls f(element index, segment) for the lane's run of up to sixteen consecutive elements of the unit.
template <typename F>
__device__ __forceinline__ void for_each_in_run(const uint64_t *lds, uint32_t n_seg, const SegUnit &q, uint32_t lane, F f)
{
    const uint32_t first = lane * kSegRun;
    if (first >= q.len) return;
    const uint32_t count = q.len - first < (uint32_t)kSegRun ? q.len - first : (uint32_t)kSegRun;
    const size_t i0 = q.start + first;
    uint32_t seg = q.single ? q.seg : segment_of_lane(lds, n_seg, i0);
    uint64_t next = seg + 1 < n_seg ? lds[seg + 1] : ~(uint64_t)0;  // the last segment has no end
    for (uint32_t i = 0; i < count; ++i) {
        const size_t idx = i0 + i;
        while (idx >= next) {  // empty segments are stepped over
            ++seg;
            next = seg + 1 < n_seg ? lds[seg + 1] : ~(uint64_t)0;
        }
        f(idx, seg);
    }
}

// An item of work is `group` consecutive units, 1 or 4 (the host takes 4 when that still leaves every wavefront of
// the chip several items).  Four units that lie inside one segment and are whole and aligned are taken at once,
// sixteen quads per lane with all their loads in flight together; otherwise each unit of the item by itself.
struct SegItem {
    size_t first_unit;   // of the item
    uint32_t units;      // that exist
    bool whole;          // the four-unit register path applies
    uint32_t seg;        // then: the segment
};

__device__ __forceinline__ SegItem open_segment_item(const uint64_t *lds, uint32_t n_seg, size_t n, size_t n_units, size_t item,
                                                     uint32_t group, uint32_t aligned, uint32_t lane)
{
    SegItem it;
    it.first_unit = item * group;
    const size_t left = n_units - it.first_unit;
    it.units = left < group ? (uint32_t)left : group;
    it.whole = false;
    it.seg = 0;
    if (group == 4 && aligned) {
        const size_t start = it.first_unit * (size_t)kSegUnit;
        if (n - start >= (size_t)(4 * kSegUnit)) {
            it.seg = segment_of_uniform(lds, n_seg, start, lane);
            it.whole = it.seg == n_seg - 1 || lds[it.seg + 1] >= start + 4 * kSegUnit;
        }
    }
    return it;
}

// Maxima of the segments into zeroed scales (non-negative binary32 numbers order like their bit patterns, so
// the pieces of a segment merge with an integer atomic max).  The sixteen wavefronts of a workgroup take sixteen
// consecutive items at a time and merge what they found through LDS first, so that a long segment costs one
// atomic per sixteen items: thousands of atomics on one address take longer than reading the array.
__global__ __launch_bounds__(kWave * kSegWaves) void k_seg_absmax(const float *__restrict__ x, size_t n,
                                                                  const uint64_t *__restrict__ bounds, uint32_t n_seg,
                                                                  size_t n_units, size_t n_items, size_t n_waves, uint32_t group,
                                                                  uint32_t aligned, float *__restrict__ scales)
{
    extern __shared__ uint64_t seg_lds[];
    __shared__ uint32_t post_seg[kSegWaves], post_max[kSegWaves];
    const uint32_t lane = threadIdx.x & 63, wave = wave_in_wg();
    load_bounds(bounds, n_seg, n, seg_lds);
    __syncthreads();
    unsigned int *sc = reinterpret_cast<unsigned int *>(scales);
    // every wavefront of the workgroup makes the same number of rounds (the barriers below)
    for (size_t base = (size_t)blockIdx.x * kSegWaves; base < n_items; base += n_waves) {
        const size_t item = base + wave;
        uint32_t my_seg = ~0u, my_max = 0;  // what this wavefront's item adds to one segment, if it is that simple
        if (item < n_items) {
            const SegItem it = open_segment_item(seg_lds, n_seg, n, n_units, item, group, aligned, lane);
            if (it.whole) {
                const v4f *p4 = reinterpret_cast<const v4f *>(x + it.first_unit * (size_t)kSegUnit);
                v4f v[4 * kSegQ];
#pragma unroll
                for (int j = 0; j < 4 * kSegQ; ++j) v[j] = ldg<1>(p4 + j * kWave + lane);
                float fm = 0.0f;
#pragma unroll
                for (int j = 0; j < 4 * kSegQ; ++j) fm = max4_abs(v[j], fm);
                my_seg = it.seg;
                my_max = wave_max_u32(f2u(fm));
            } else {
                for (uint32_t r = 0; r < it.units; ++r) {
                    const SegUnit q = open_segment_unit(seg_lds, n_seg, n, it.first_unit + r, lane);
                    if (q.single && q.len == (uint32_t)kSegUnit && aligned) {
                        const v4f *p4 = reinterpret_cast<const v4f *>(x + q.start);
                        float fm = 0.0f;
#pragma unroll
                        for (int j = 0; j < kSegQ; ++j) fm = max4_abs(ldg<1>(p4 + j * kWave + lane), fm);
                        const uint32_t m = wave_max_u32(f2u(fm));
                        if (group == 1) {  // the item is this unit: merged with the workgroup's other items below
                            my_seg = q.seg;
                            my_max = m;
                        } else if (lane == 0 && m != 0) {
                            atomicMax(sc + q.seg, m);
                        }
                    } else {
                        uint32_t run = 0, run_seg = 0;
                        for_each_in_run(seg_lds, n_seg, q, lane, [&](size_t idx, uint32_t seg) {
                            if (seg != run_seg) {
                                if (run != 0) atomicMax(sc + run_seg, run);
                                run = 0;
                                run_seg = seg;
                            }
                            const uint32_t a = abs_bits(x[idx]);
                            run = run > a ? run : a;
                        });
                        if (run != 0) atomicMax(sc + run_seg, run);
                    }
                }
            }
        }
        if (lane == 0) {
            post_seg[wave] = my_seg;
            post_max[wave] = my_max;
        }
        __syncthreads();
        if (wave == 0 && lane < (uint32_t)kSegWaves) {
            // lane l speaks for the wavefronts that posted the same segment as wavefront l, if it is the first of them
            const uint32_t s = post_seg[lane];
            uint32_t m = 0;
            bool first = true;
            for (uint32_t j = 0; j < (uint32_t)kSegWaves; ++j) {
                if (post_seg[j] == s) {
                    if (j < lane) first = false;
                    m = m > post_max[j] ? m : post_max[j];
                }
            }
            if (first && s != ~0u && m != 0) atomicMax(sc + s, m);
        }
        __syncthreads();  // the posts are rewritten in the next round
    }
}

// Compression with the segments' scales (computed by k_seg_absmax or handed in).
template <bool REMAP>
__global__ __launch_bounds__(kWave * kSegWaves) void k_seg_encode(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                                  size_t n, const uint64_t *__restrict__ bounds, uint32_t n_seg,
                                                                  size_t n_units, size_t n_waves, uint32_t aligned,
                                                                  const float *__restrict__ scales, uint8_t *__restrict__ codes)
{
    extern __shared__ uint64_t seg_lds[];  // the bounds (n_seg + 1 entries, rounded up to an even count of words), then the search table
    const uint32_t lane = threadIdx.x & 63;
    load_bounds(bounds, n_seg, n, seg_lds);
    Search sr = load_bucket_table(tab, reinterpret_cast<uint32_t *>(seg_lds + n_seg + 1), kWave * kSegWaves);
    sr.marks = REMAP;
    __syncthreads();
    for (size_t u = first_unit(kSegWaves); u < n_units; u += n_waves) {
        const SegUnit q = open_segment_unit(seg_lds, n_seg, n, u, lane);
        if (q.single && q.len == (uint32_t)kSegUnit && aligned) {
            const v4f *p4 = reinterpret_cast<const v4f *>(x + q.start);
            v4f v[kSegQ];
#pragma unroll
            for (int j = 0; j < kSegQ; ++j) v[j] = ldg<1>(p4 + j * kWave + lane);
            const float s = scales[q.seg];
            const float d = s == 0.0f ? 1.0f : s;
            const float r = 1.0f / d;
            const bool recip = reciprocal_ok(d);
            uint32_t cw[kSegQ];
            encode_quads<true, kSegQ>(sr, v, d, r, recip, cw);
            uint32_t *c4 = reinterpret_cast<uint32_t *>(codes + q.start);
#pragma unroll
            for (int j = 0; j < kSegQ; ++j) stg<1>(c4 + j * kWave + lane, cw[j]);
        } else {
            uint32_t cur = ~0u;
            float d = 1.0f, r = 1.0f;
            bool recip = true;
            for_each_in_run(seg_lds, n_seg, q, lane, [&](size_t idx, uint32_t seg) {
                if (seg != cur) {
                    cur = seg;
                    const float s = scales[seg];
                    d = s == 0.0f ? 1.0f : s;
                    r = 1.0f / d;
                    recip = reciprocal_ok(d);
                }
                codes[idx] = (uint8_t)encode_one<false>(sr, x[idx], d, r, recip);
            });
        }
    }
}

// Decompression with the segments' scales.
__global__ __launch_bounds__(kWave * kSegWaves) void k_seg_decode(const uint32_t *__restrict__ tab, const uint8_t *__restrict__ codes,
                                                                  const float *__restrict__ scales, size_t n,
                                                                  const uint64_t *__restrict__ bounds, uint32_t n_seg,
                                                                  size_t n_units, size_t n_waves, uint32_t aligned,
                                                                  float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint64_t seg_lds[];
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    load_bounds(bounds, n_seg, n, seg_lds);
    load_lut(tab, lut);
    __syncthreads();
    for (size_t u = first_unit(kSegWaves); u < n_units; u += n_waves) {
        const SegUnit q = open_segment_unit(seg_lds, n_seg, n, u, lane);
        if (q.single && q.len == (uint32_t)kSegUnit && aligned) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(codes + q.start);
            uint32_t w[kSegQ];
#pragma unroll
            for (int j = 0; j < kSegQ; ++j) w[j] = ldg<1>(c4 + j * kWave + lane);
            const float s = scales[q.seg];
            v4f *o4 = reinterpret_cast<v4f *>(out + q.start);
#pragma unroll
            for (int j = 0; j < kSegQ; ++j) {
                v4f r;
                r.x = lut_at<0>(lut, w[j], lane4) * s;
                r.y = lut_at<1>(lut, w[j], lane4) * s;
                r.z = lut_at<2>(lut, w[j], lane4) * s;
                r.w = lut_at<3>(lut, w[j], lane4) * s;
                stg<2>(o4 + j * kWave + lane, r);
            }
        } else {
            uint32_t cur = ~0u;
            float s = 0.0f;
            for_each_in_run(seg_lds, n_seg, q, lane, [&](size_t idx, uint32_t seg) {
                if (seg != cur) {
                    cur = seg;
                    s = scales[seg];
                }
                out[idx] = lut_code(lut, codes[idx], lane4) * s;
            });
        }
    }
}

// Decompression of K workers' buffers and their average (optionally with a local fp32 array as the first term)
// with the segments' scales: the ordered sum of the other averaging kernels (product and sum rounded separately,
// workers in index order, then the division by the number of terms), any number of workers, four at a time in
// flight on the register path.
__global__ __launch_bounds__(kWave * kSegWaves) void k_seg_avg(const uint32_t *__restrict__ tab, WorkerPtrs p, int K,
                                                               const float *__restrict__ local, size_t n,
                                                               const uint64_t *__restrict__ bounds, uint32_t n_seg,
                                                               size_t n_units, size_t n_waves, uint32_t aligned,
                                                               float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint64_t seg_lds[];
    const uint32_t lane = threadIdx.x & 63, lane4 = lane * 4;
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    load_bounds(bounds, n_seg, n, seg_lds);
    load_lut(tab, lut);
    __syncthreads();
    constexpr int kAhead = 4;  // workers whose code words are requested together
    for (size_t u = first_unit(kSegWaves); u < n_units; u += n_waves) {
        const SegUnit q = open_segment_unit(seg_lds, n_seg, n, u, lane);
        if (q.single && q.len == (uint32_t)kSegUnit && aligned) {
            v4f acc[kSegQ];
            if (local) {  // the sum starts at +0: a local -0 becomes +0
                const v4f *l4 = reinterpret_cast<const v4f *>(local + q.start);
#pragma unroll
                for (int j = 0; j < kSegQ; ++j) {
                    const v4f l = ldg<1>(l4 + j * kWave + lane);
                    acc[j] = v4f{0.0f + l.x, 0.0f + l.y, 0.0f + l.z, 0.0f + l.w};
                }
            } else {
#pragma unroll
                for (int j = 0; j < kSegQ; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
            }
            for (int k0 = 0; k0 < K; k0 += kAhead) {
                uint32_t w[kAhead][kSegQ];
                float sc[kAhead];
#pragma unroll
                for (int c = 0; c < kAhead; ++c) {
                    const int k = k0 + c < K ? k0 + c : K - 1;  // a place past the last worker repeats it and is not added
                    const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k] + q.start);
                    sc[c] = p.scales[k][q.seg];
#pragma unroll
                    for (int j = 0; j < kSegQ; ++j) w[c][j] = ldg<1>(c4 + j * kWave + lane);
                }
#pragma unroll
                for (int c = 0; c < kAhead; ++c) {
                    if (k0 + c < K) {
#pragma unroll
                        for (int j = 0; j < kSegQ; ++j) {
                            acc[j].x = acc[j].x + lut_at<0>(lut, w[c][j], lane4) * sc[c];
                            acc[j].y = acc[j].y + lut_at<1>(lut, w[c][j], lane4) * sc[c];
                            acc[j].z = acc[j].z + lut_at<2>(lut, w[c][j], lane4) * sc[c];
                            acc[j].w = acc[j].w + lut_at<3>(lut, w[c][j], lane4) * sc[c];
                        }
                    }
                }
            }
            v4f *o4 = reinterpret_cast<v4f *>(out + q.start);
#pragma unroll
            for (int j = 0; j < kSegQ; ++j)
                stg<2>(o4 + j * kWave + lane, v4f{mean_of(acc[j].x), mean_of(acc[j].y), mean_of(acc[j].z), mean_of(acc[j].w)});
        } else {
            for_each_in_run(seg_lds, n_seg, q, lane, [&](size_t idx, uint32_t seg) {
                float a = 0.0f;
                if (local) a = a + local[idx];
                for (int k = 0; k < K; ++k) a = a + lut_code(lut, p.codes[k][idx], lane4) * p.scales[k][seg];
                out[idx] = mean_of(a);
            });
        }
    }
}

}  // namespace
