// dq8 kernels for one buffer: block maxima, compression, decompression, and the calibration copy.
#pragma once
#include "dq8_device.hpp"

namespace {

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
    // Units of 8192 and 16384 elements serve every block length above 4096: a short block leaves whole rows
    // of a unit empty, which are neither loaded nor quantised.
    static constexpr bool kSkipRows = WPB > 1 && QL > 4;

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
                if (kSkipRows && it * TEAM > last) {  // the same for the whole team: a row past the end of the unit
                    sl.v[it] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
                    continue;
                }
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
            // quads whose table lookups are issued together; the team variant runs six teams per compute unit
            // and has no registers to spare for that
            constexpr int G = WPB > 1 ? 1 : (Q < 4 ? Q : 4);
#pragma unroll
            for (int g = 0; g < Q; g += G) {
                if (kSkipRows && g * TEAM >= nq) continue;
                v4f vv[G];
                uint32_t cw[G];
#pragma unroll
                for (int it = 0; it < G; ++it) vv[it] = sl.v[g + it];
                encode_quads<FASTDIV, G>(sr, vv, d, r, recip, cw);
#pragma unroll
                for (int it = 0; it < G; ++it)
                    if ((g + it) * TEAM + tl < nq) stg<NT>(c4 + (g + it) * TEAM + tl, cw[it]);
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

// Compression of whole, aligned blocks of 4096 elements: the common case of k_encode<4, 4, NT, true,
// FASTDIV> (a team of four wavefronts per block, maximum and quantisation from registers) with
// nothing else in the loop.  Block b starts at element 4096 b, x is 16-byte and codes 4-byte
// aligned, so unit geometry is a multiplication and there is no slow path to branch around.
// A ragged last block of tail_len elements is done by the last workgroup after its loop.
// REMAP says whether code bytes of the data type can carry marks (see fix_marked_codes): known at compile time,
// so the test for it drops out of the loop.
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
        uint32_t cw[Q];
        encode_quads<FASTDIV, Q>(sr, v, d, r, recip, cw);
#pragma unroll
        for (int it = 0; it < Q; ++it) stg_at<NT>(c4, it * kWg + tl, cw[it]);
    };
    uint32_t u = blockIdx.x;
    v4f a[Q], b[Q];
    if (u < n_full) fetch(u, a);  // the first loads are in flight while the table is copied
    sr = load_bucket_table(tab, lds + kTeamSlots);
    sr.marks = REMAP;  // known at compile time: no test for marked code bytes in the loop
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

// Compression of blocks of up to QL * 256 elements, one wavefront per block: k_encode_long without the exchange
// between wavefronts.  Blocks are whole quads (bq of them), x is 16-byte and codes 4-byte aligned; a lane whose
// quad lies past the end of the block loads the block's last quad instead and stores nothing; the last block
// may be shorter (tail_q quads, 0: none).  Wavefront w of the grid takes blocks w, w + n_waves, ...
template <int QL, int NT, int WPW, bool REMAP>
__global__ __launch_bounds__(kWave * WPW) void k_encode_wave(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                            uint32_t n_units, uint32_t n_waves, uint32_t bq,
                                                            uint32_t tail_q, float *__restrict__ scales,
                                                            uint8_t *__restrict__ codes)
{
    constexpr int Q = QL;
    constexpr int G = Q < 4 ? Q : 4;  // quads whose table lookups are issued together
    static_assert(Q % G == 0, "whole groups of quads");
    extern __shared__ uint32_t lds[];  // the bucket table
    const uint32_t lane = threadIdx.x & 63;
    Search sr;
    auto quads_of = [&](uint32_t u) { return (tail_q != 0 && u == n_units - 1) ? tail_q : bq; };
    auto fetch = [&](uint32_t u, v4f(&v)[Q]) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x) + (size_t)u * bq;
        const uint32_t last = quads_of(u) - 1;
#pragma unroll
        for (int it = 0; it < Q; ++it) {
            const uint32_t q = it * kWave + lane;
            v[it] = ldg_at<NT>(p4, q < last ? q : last);
        }
    };
    auto process = [&](uint32_t u, v4f(&v)[Q]) {
        float fm = 0.0f;
#pragma unroll
        for (int it = 0; it < Q; ++it) fm = max4_abs(v[it], fm);
        const float s = u2f(wave_max_u32(f2u(fm)));
        if (lane == 0) scales[u] = s;
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes) + (size_t)u * bq;
        const uint32_t nq = quads_of(u);
#pragma unroll
        for (int g = 0; g < Q; g += G) {
            v4f vv[G];
            uint32_t cw[G];
#pragma unroll
            for (int it = 0; it < G; ++it) vv[it] = v[g + it];
            encode_quads<true, G>(sr, vv, d, r, recip, cw);
#pragma unroll
            for (int it = 0; it < G; ++it) {
                const uint32_t q = (g + it) * kWave + lane;
                if (q < nq) stg_at<NT>(c4, q, cw[it]);
            }
        }
    };
    uint32_t u = (uint32_t)first_unit(WPW);
    v4f a[Q], b[Q];
    if (u < n_units) fetch(u, a);  // the first loads are in flight while the table is copied
    sr = load_bucket_table(tab, lds, kWave * WPW);
    sr.marks = REMAP;  // known at compile time: no test for marked code bytes in the loop
    __syncthreads();
    // steady state as in k_encode_full: the next block's loads are issued unconditionally before the work on
    // the current one
    if (u < n_units) {
        for (;;) {
            uint32_t nx = u + n_waves;
            if (!(nx < n_units)) {
                process(u, a);
                break;
            }
            fetch(nx, b);
            process(u, a);
            u = nx;
            nx = u + n_waves;
            if (!(nx < n_units)) {
                process(u, b);
                break;
            }
            fetch(nx, a);
            process(u, b);
            u = nx;
        }
    }
}

// Decompression with units that do not follow the blocks: unit u is quads [u Q 64, (u + 1) Q 64) of the array
// (a quad = 4 consecutive elements; blocks are whole quads, bq of them, so a quad never straddles two blocks),
// whatever the block length.  The host picks Q and NS with Q 64 <= (NS - 1) bq: a unit then touches at most NS
// blocks, whose scales are NS scalar loads (indices clamped to the last block), and every quad selects its own
// by comparing its offset from the start of the unit's first block with bq, 2 bq, ...  The block index and
// offset of a wavefront's unit advance by the same step every iteration (step_b blocks and step_r < bq
// quads), so there is one division per wavefront.  out is 16-byte, codes 4-byte aligned; the last unit may be
// short (a lane past the end repeats the last code word's load and stores nothing); `left` elements after the
// last whole quad (they belong to the last block) are done one by one by the wavefront that has the last unit.
template <int Q, int NS, int NT, int WPW>
__global__ __launch_bounds__(kWave * WPW) void k_decode_flat(const uint32_t *__restrict__ tab, const uint8_t *__restrict__ codes,
                                                            const float *__restrict__ scales, uint64_t nq, uint32_t left,
                                                            uint32_t bq, uint64_t nb, uint64_t n_units, uint32_t n_waves,
                                                            uint64_t step_b, uint32_t step_r, float *__restrict__ out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    constexpr uint32_t UQ = Q * kWave;  // quads per unit
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t lane4 = lane * 4;
    uint64_t u = first_unit(WPW);
    uint64_t b0 = (u * UQ) / bq;               // block of the unit's first quad
    uint32_t r0 = (uint32_t)((u * UQ) % bq);   // and that quad's offset in it
    uint32_t w[Q], len = 0;
    float sc[NS];
    auto open_unit = [&](uint64_t uu, uint64_t bb) {
        const uint32_t *c4 = reinterpret_cast<const uint32_t *>(codes) + uu * UQ;
        const uint64_t rest = nq - uu * UQ;
        len = rest < UQ ? (uint32_t)rest : UQ;
        const uint32_t last = len - 1;
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint32_t i = j * kWave + lane;
            w[j] = ldg_at<NT>(c4, i < last ? i : last);
        }
#pragma unroll
        for (int t = 0; t < NS; ++t) sc[t] = scales[bb + t < nb ? bb + t : nb - 1];
    };
    if (u < n_units) open_unit(u, b0);  // the first loads are in flight while the table is built
    load_lut(tab, lut);
    __syncthreads();
    while (u < n_units) {
        uint32_t cur[Q];
#pragma unroll
        for (int j = 0; j < Q; ++j) cur[j] = w[j];
        float cs[NS];
#pragma unroll
        for (int t = 0; t < NS; ++t) cs[t] = sc[t];
        const uint32_t nqu = len, base = r0 + lane;
        v4f *o4 = reinterpret_cast<v4f *>(out) + u * UQ;
        const bool last_unit = u == n_units - 1;
        const uint64_t last_block = nb - 1;
        u += n_waves;
        b0 += step_b;
        r0 += step_r;
        if (r0 >= bq) {
            r0 -= bq;
            b0 += 1;
        }
        if (u < n_units) open_unit(u, b0);
#pragma unroll
        for (int j = 0; j < Q; ++j) {
            const uint32_t o = base + j * kWave;
            float s = cs[0];
#pragma unroll
            for (int t = 1; t < NS; ++t) s = o >= (uint32_t)t * bq ? cs[t] : s;
            v4f r;
            r.x = lut_at<0>(lut, cur[j], lane4) * s;
            r.y = lut_at<1>(lut, cur[j], lane4) * s;
            r.z = lut_at<2>(lut, cur[j], lane4) * s;
            r.w = lut_at<3>(lut, cur[j], lane4) * s;
            if (j * kWave + lane < nqu) stg<NT>(o4 + j * kWave + lane, r);
        }
        if (last_unit && lane < left) {
            const uint64_t e = nq * 4 + lane;
            out[e] = lut_code(lut, codes[e], lane4) * scales[last_block];
        }
    }
    // an array shorter than a quad has no unit at all
    if (n_units == 0 && blockIdx.x == 0 && wave_in_wg() == 0 && lane < left) out[lane] = lut_code(lut, codes[lane], lane4) * scales[0];
}

// Compression of blocks of up to 16384 elements from one read of x: the scheme of k_encode_full with QPL
// quads per lane (a team of four wavefronts holds up to QPL * 1024 elements) and a block length given
// at run time.  Blocks are whole quads (bq of them) and x is 16-byte, codes 4-byte aligned, so every block
// starts on aligned addresses.  A lane whose quad lies past the end of the block loads the block's last quad
// instead (an unconditional load of valid memory: the maximum does not change and the lane stores nothing).
// The last block may be shorter (tail_q quads, 0: none): it is one more unit, with its own length.
template <int QPL, int NT, bool REMAP>
__global__ __launch_bounds__(kWg) void k_encode_long(const uint32_t *__restrict__ tab, const float *__restrict__ x,
                                                    uint32_t n_units, uint32_t n_teams, uint32_t bq, uint32_t tail_q,
                                                    float *__restrict__ scales, uint8_t *__restrict__ codes)
{
    constexpr int Q = QPL;
    constexpr int G = Q < 4 ? Q : (Q % 4 == 0 ? 4 : 2);  // quads whose table lookups are issued together
    static_assert(Q % G == 0, "whole groups of quads");
    extern __shared__ uint32_t lds[];
    uint32_t *slots = lds;  // kTeamSlots words, then the bucket table
    const uint32_t lane = threadIdx.x & 63, wave = wave_in_wg(), tl = threadIdx.x;
    uint32_t phase = 0;
    Search sr;
    auto quads_of = [&](uint32_t u) { return (tail_q != 0 && u == n_units - 1) ? tail_q : bq; };
    auto fetch = [&](uint32_t u, v4f(&v)[Q]) {
        const v4f *p4 = reinterpret_cast<const v4f *>(x) + (size_t)u * bq;
        const uint32_t last = quads_of(u) - 1;
#pragma unroll
        for (int it = 0; it < Q; ++it) {
            const uint32_t q = it * kWg + tl;
            v[it] = ldg_at<NT>(p4, q < last ? q : last);
        }
    };
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
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes) + (size_t)u * bq;
        const uint32_t nq = quads_of(u);
#pragma unroll
        for (int g = 0; g < Q; g += G) {
            v4f vv[G];
            uint32_t cw[G];
#pragma unroll
            for (int it = 0; it < G; ++it) vv[it] = v[g + it];
            encode_quads<true, G>(sr, vv, d, r, recip, cw);
#pragma unroll
            for (int it = 0; it < G; ++it) {
                const uint32_t q = (g + it) * kWg + tl;
                if (q < nq) stg_at<NT>(c4, q, cw[it]);
            }
        }
    };
    uint32_t u = blockIdx.x;
    v4f a[Q], b[Q];
    if (u < n_units) fetch(u, a);  // the first loads are in flight while the table is copied
    sr = load_bucket_table(tab, lds + kTeamSlots);
    sr.marks = REMAP;  // known at compile time: no test for marked code bytes in the loop
    __syncthreads();
    // steady state as in k_encode_full: the next block's loads are issued unconditionally before the work on
    // the current one
    if (u < n_units) {
        for (;;) {
            uint32_t nx = u + n_teams;
            if (!(nx < n_units)) {
                process(u, a);
                break;
            }
            fetch(nx, b);
            process(u, a);
            u = nx;
            nx = u + n_teams;
            if (!(nx < n_units)) {
                process(u, b);
                break;
            }
            fetch(nx, a);
            process(u, b);
            u = nx;
        }
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

}  // namespace
