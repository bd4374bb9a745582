// dq8 kernels that decompress K workers' buffers and average them into an fp32 array.
#pragma once
#include "dq8_device.hpp"

namespace {

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
                    for (int k0 = 0; k0 < K; k0 += 4) {  // four workers' loads in flight at a time
                        uint32_t ww[4];
                        float ss[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int k = k0 + i < K ? k0 + i : K - 1;  // past the last worker: a valid, unused load
                            ww[i] = ldg<NT>(reinterpret_cast<const uint32_t *>(p.codes[k] + un.start) + q);
                            ss[i] = p.scales[k][un.block];
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (k0 + i < K) {
                                a.x = a.x + lut_at<0>(lut, ww[i], lane4) * ss[i];
                                a.y = a.y + lut_at<1>(lut, ww[i], lane4) * ss[i];
                                a.z = a.z + lut_at<2>(lut, ww[i], lane4) * ss[i];
                                a.w = a.w + lut_at<3>(lut, ww[i], lane4) * ss[i];
                            }
                        }
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

// K-way decode-and-average of whole, aligned units, K up to 12 (fixed at compile time; above 8 with Q = 1): the common case of
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
    static_assert(KT >= 1 && KT <= 12 && KT * Q <= 32, "up to twelve workers and 32 code words per lane and set");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    constexpr float fk = (float)(KT + (LOCAL ? 1 : 0));
    constexpr int terms = KT + (LOCAL ? 1 : 0);
    constexpr bool pow2 = (terms & (terms - 1)) == 0;
    constexpr float rk = 1.0f / fk;  // acc * (1 / K) equals acc / K exactly for a power of two
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
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

// k_decode_avg_full for block lengths that are whole quads (bq of them, at least as many as a unit has, or
// exactly half as many) but not a power-of-two number of units: unit u is still quads [u Q 64, (u + 1) Q 64) of
// the array, so it touches at most two blocks.  Both blocks' scales travel with the unit's code words (two scalar loads per worker, the second
// index clamped to the last block) and every quad selects by comparing its offset from the start of the first
// block with bq.  The block index b and offset r of a wavefront's units advance by the same step every
// iteration (step_b blocks and step_r < bq quads): one division per wavefront.
struct FlatGeom {
    uint32_t bq, last_block, step_b, step_r;
};

template <int KT, int NT, int WPW, bool LOCAL>
__global__ __launch_bounds__(kWave * WPW) void k_decode_avg_flat(const uint32_t *__restrict__ tab, WorkerPtrs p,
                                                                const float *__restrict__ local, uint32_t n_full,
                                                                uint32_t n_waves, FlatGeom g, uint32_t tail_len,
                                                                float *__restrict__ out)
{
    static_assert(KT >= 1 && KT <= 8, "unrolled for up to eight workers");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int Q = 2;
    constexpr int U = Q * 4 * kWave;
    constexpr uint32_t UQ = Q * kWave;
    constexpr float fk = (float)(KT + (LOCAL ? 1 : 0));
    constexpr int terms = KT + (LOCAL ? 1 : 0);
    constexpr bool pow2 = (terms & (terms - 1)) == 0;
    constexpr float rk = 1.0f / fk;  // acc * (1 / K) equals acc / K exactly for a power of two
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    struct Slot {
        uint32_t w[KT][Q];
        float s0[KT], s1[KT];
        uint32_t r;
        v4f loc[LOCAL ? Q : 1];
    };
    uint32_t fb = 0, fr = 0;  // block and offset of the first quad of the next unit to fetch
    auto fetch = [&](uint32_t u, Slot &sl) {
        if (LOCAL) {
            const v4f *l4 = reinterpret_cast<const v4f *>(local) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) sl.loc[j] = ldg_at<NT>(l4, j * kWave + lane);
        }
        const uint32_t b1 = fb < g.last_block ? fb + 1 : g.last_block;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            sl.s0[k] = p.scales[k][fb];
            sl.s1[k] = p.scales[k][b1];
        }
        sl.r = fr;
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k]) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) sl.w[k][j] = ldg_at<NT>(c4, j * kWave + lane);
        }
        fb += g.step_b;
        fr += g.step_r;
        if (fr >= g.bq) {
            fr -= g.bq;
            fb += 1;
        }
    };
    auto process = [&](uint32_t u, Slot &sl) {
        float a0[KT], a1[KT];
#pragma unroll
        for (int k = 0; k < KT; ++k) {
            a0[k] = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(sl.s0[k])));
            a1[k] = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(sl.s1[k])));
        }
        const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)sl.r) + lane;
        v4f *o4 = reinterpret_cast<v4f *>(out) + (size_t)u * (U / 4);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const bool second = base + j * kWave >= g.bq;  // this quad lies in the unit's second block
            v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
            if (LOCAL) {  // the sum starts at +0: a local -0 becomes +0
                a.x = a.x + sl.loc[j].x;
                a.y = a.y + sl.loc[j].y;
                a.z = a.z + sl.loc[j].z;
                a.w = a.w + sl.loc[j].w;
            }
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const float sc = second ? a1[k] : a0[k];
                a.x = a.x + lut_at<0>(lut, sl.w[k][j], lane4) * sc;
                a.y = a.y + lut_at<1>(lut, sl.w[k][j], lane4) * sc;
                a.z = a.z + lut_at<2>(lut, sl.w[k][j], lane4) * sc;
                a.w = a.w + lut_at<3>(lut, sl.w[k][j], lane4) * sc;
            }
            a.x = mean_of(a.x);
            a.y = mean_of(a.y);
            a.z = mean_of(a.z);
            a.w = mean_of(a.w);
            stg<NT>(o4 + j * kWave + lane, a);
        }
    };
    uint32_t u = (uint32_t)first_unit(WPW);
    {
        const uint64_t q0 = (uint64_t)u * UQ;
        fb = (uint32_t)(q0 / g.bq);
        fr = (uint32_t)(q0 % g.bq);
    }
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
        const size_t B = (size_t)g.bq * 4;
        for (uint32_t i = lane; i < tail_len; i += kWave) {
            const size_t blk = (start + i) / B;
            float acc = 0.0f;
            if (LOCAL) acc = acc + local[start + i];
#pragma unroll
            for (int k = 0; k < KT; ++k) acc = acc + lut_code(lut, p.codes[k][start + i], lane4) * p.scales[k][blk];
            out[start + i] = mean_of(acc);
        }
    }
}

// K-way decode-and-average of whole, aligned units for any K (and an optional local fp32 first term): the
// workers are taken CH at a time (the host picks the CH <= 8 that leaves the fewest empty places in the last
// chunk).  Work items are (unit, chunk of CH workers) pairs in order; the code
// words and scales of the next item are requested before the current one is added to the running sums, which
// stay in registers from a unit's first chunk to its last.  Every request is unconditional (the item after
// the last one is the last one again, a worker index past K - 1 is K - 1 with scale 0), so the compiler waits
// for exactly the loads an item needs.  Geometry as in k_decode_avg_full.
// FLAT: the geometry of k_decode_avg_flat instead (blocks of whole quads, at most two per unit; Q = 2): every
// place of a chunk carries both blocks' scales, and the block and offset of a unit advance with the unit.
template <int CH, int Q, int NT, int WPW, bool FLAT>
__global__ __launch_bounds__(kWave * WPW) void k_decode_avg_chunks(const uint32_t *__restrict__ tab, WorkerPtrs p, int K,
                                                                  const float *__restrict__ local, uint32_t n_full,
                                                                  uint32_t n_waves, uint32_t block_shift, FlatGeom g,
                                                                  uint32_t tail_len, float *__restrict__ out)
{
    static_assert(!FLAT || Q == 2, "the position-based geometry is laid out for two code words per lane");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr int U = Q * 4 * kWave;
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    const uint32_t n_chunks = (uint32_t)(K + CH - 1) / CH;  // 0 when K == 0: the local term alone
    struct Slot {
        uint32_t w[CH][Q];
        float sw[CH];
        float sw1[FLAT ? CH : 1];
        uint32_t r;
    };
    // FLAT: block and offset of the first quad of the unit whose chunks are being fetched
    uint32_t fb = 0, fr = 0;
    auto fetch = [&](uint32_t u, uint32_t c, Slot &sl) {
        const uint32_t b0 = FLAT ? fb : (u >> block_shift);
        const uint32_t b1 = FLAT ? (fb < g.last_block ? fb + 1 : g.last_block) : 0;
        sl.r = fr;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int k = (int)(c * CH) + i;
            const bool empty = !(k < K);  // an empty place of the last chunk: worker K - 1 again, with scale 0
            k = empty ? K - 1 : k;
            const float s = p.scales[k][b0];
            sl.sw[i] = empty ? 0.0f : s;
            if (FLAT) {
                const float s1 = p.scales[k][b1];
                sl.sw1[i] = empty ? 0.0f : s1;
            }
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k]) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) sl.w[i][j] = ldg_at<NT>(c4, j * kWave + lane);
        }
    };
    v4f acc[Q];
    auto start_unit = [&](uint32_t u) {
        if (local) {  // not prefetched: once per unit
            const v4f *l4 = reinterpret_cast<const v4f *>(local) + (size_t)u * (U / 4);
#pragma unroll
            for (int j = 0; j < Q; ++j) {  // the sum starts at +0: a local -0 becomes +0
                const v4f l = ldg_at<NT>(l4, j * kWave + lane);
                acc[j] = v4f{0.0f + l.x, 0.0f + l.y, 0.0f + l.z, 0.0f + l.w};
            }
        } else {
#pragma unroll
            for (int j = 0; j < Q; ++j) acc[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        }
    };
    auto finish_unit = [&](uint32_t u) {
        v4f *o4 = reinterpret_cast<v4f *>(out) + (size_t)u * (U / 4);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            v4f a = acc[j];
            a.x = mean_of(a.x);
            a.y = mean_of(a.y);
            a.z = mean_of(a.z);
            a.w = mean_of(a.w);
            stg<NT>(o4 + j * kWave + lane, a);
        }
    };
    // Adds chunk c of unit u from its slot; opens the unit's sums at its first chunk and stores the means at its last.
    auto process = [&](uint32_t u, uint32_t c, const Slot &sl) {
        if (c == 0) start_unit(u);
        // No branch around an empty place: its scale is 0, the product is a zero of either sign, and adding
        // that changes nothing (a running sum that starts at +0 is never -0).
        const uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)sl.r) + lane;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const float s0 = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(sl.sw[i])));
            const float s1 = FLAT ? u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(sl.sw1[i]))) : 0.0f;
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const float s = (FLAT && base + j * kWave >= g.bq) ? s1 : s0;  // the quad lies in the unit's second block
                acc[j].x = acc[j].x + lut_at<0>(lut, sl.w[i][j], lane4) * s;
                acc[j].y = acc[j].y + lut_at<1>(lut, sl.w[i][j], lane4) * s;
                acc[j].z = acc[j].z + lut_at<2>(lut, sl.w[i][j], lane4) * s;
                acc[j].w = acc[j].w + lut_at<3>(lut, sl.w[i][j], lane4) * s;
            }
        }
        if (c + 1 == n_chunks) finish_unit(u);
    };
    // The item after (u, c), and whether there is one; without one the same item again.
    auto advance = [&](uint32_t &u, uint32_t &c) {
        if (c + 1 < n_chunks) {
            ++c;
            return true;
        }
        if (u + n_waves < n_full) {
            u += n_waves;
            c = 0;
            if (FLAT) {  // the fetches that follow belong to that unit
                fb += g.step_b;
                fr += g.step_r;
                if (fr >= g.bq) {
                    fr -= g.bq;
                    fb += 1;
                }
            }
            return true;
        }
        return false;
    };
    uint32_t u = (uint32_t)first_unit(WPW), c = 0;
    if (FLAT) {
        const uint64_t q0 = (uint64_t)u * (Q * kWave);
        fb = (uint32_t)(q0 / g.bq);
        fr = (uint32_t)(q0 % g.bq);
    }
    Slot a, b;
    const bool any = u < n_full && n_chunks > 0;
    if (any) fetch(u, 0, a);  // the first loads are in flight while the table is built
    load_lut(tab, lut);
    __syncthreads();
    if (any) {
        for (;;) {
            uint32_t un = u, cn = c;
            bool more = advance(un, cn);
            fetch(un, cn, b);
            process(u, c, a);
            if (!more) break;
            u = un;
            c = cn;
            more = advance(un, cn);
            fetch(un, cn, a);
            process(u, c, b);
            if (!more) break;
            u = un;
            c = cn;
        }
    } else if (n_chunks == 0) {  // K == 0: the local values alone
        for (; u < n_full; u += n_waves) {
            start_unit(u);
            finish_unit(u);
        }
    }
    if (tail_len != 0 && blockIdx.x == gridDim.x - 1 && wave_in_wg() == 0) {
        const size_t start = (size_t)n_full * U;
        for (uint32_t i = lane; i < tail_len; i += kWave) {
            const size_t blk = FLAT ? (start + i) / ((size_t)g.bq * 4) : (size_t)(n_full >> block_shift);
            float s = 0.0f;
            if (local) s = s + local[start + i];
            for (int k = 0; k < K; ++k) s = s + lut_code(lut, p.codes[k][start + i], lane4) * p.scales[k][blk];
            out[start + i] = mean_of(s);
        }
    }
}

}  // namespace
