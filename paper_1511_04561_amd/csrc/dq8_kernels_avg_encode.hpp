// dq8 kernels that average K workers' buffers in registers and store the mean and / or compress it
// again (the second round of the gradient exchange).
#pragma once
#include <type_traits>
#include <utility>

#include "dq8_device.hpp"

namespace {

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
            // (one test per element: with one test around all the multiplications and one around all the divisions
            // the compiler interleaves them and spills a hundred registers in the 16-quad form of this kernel)
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
                constexpr int G = Q < 4 ? Q : 4;  // quads whose table lookups are issued together
#pragma unroll
                for (int g = 0; g < Q; g += G) {
                    v4f vv[G];
                    uint32_t cw[G];
#pragma unroll
                    for (int j = 0; j < G; ++j) vv[j] = acc[g + j];
                    encode_quads<FASTDIV, G>(sr, vv, d, r, recip, cw);
#pragma unroll
                    for (int j = 0; j < G; ++j)
                        if (!RAGGED || (g + j) * kWave + lane < nq) stg<1>(c4 + (g + j) * kWave + lane, cw[j]);
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

// Average-then-compress for scale blocks of 4097 .. 16384 elements: the scheme of k_avg_block with a workgroup of
// eight wavefronts per block (two such workgroups share a compute unit: each holds the 64 KiB decode table).
// Every lane holds QL quads of running sums (quad it * 512 + t of the block for thread t) and the block maximum of
// the means is a wave reduction plus one LDS exchange between the eight wavefronts.  Blocks are handed out by
// position (block b to workgroup b mod n_teams), so every wavefront of a workgroup walks the same blocks and meets
// the same barriers.
//
// The workgroup's work is one sequence of (block, worker) pairs: all workers of its first block, then all workers
// of its second block, and so on.  NB register sets of code words rotate over that sequence: the pair that is
// being added uses one set and the NB - 1 pairs after it are in flight, across the end of a block as well, so
// the loads for the next block travel while the maximum is exchanged and the means are compressed.  Every step
// issues exactly one set of loads and consumes exactly one, with no branch around either: the compiler then
// knows how many loads are outstanding at every point and waits for the oldest set only.  For that
//  - the number of workers is padded to a multiple of NB: a place without a worker repeats worker K - 1 (a hit in
//    the cache) and is added with scale 0 (the product is a zero, and adding a zero to a sum that started at +0
//    leaves it unchanged);
//  - the worker's scale for the block is loaded with its code words, one more load of the set (requested at the
//    start of a block it would be the wavefront's youngest load, and waiting for it would drain everything);
//  - a place past the workgroup's last block repeats its last block (valid memory, result unused);
//  - a lane whose quad lies past the end of a block loads the block's last quad and stores nothing.
// `aligned` (from the host): every buffer allows 32-bit accesses to the codes and 128-bit ones to local at
// every block start, and there is at least one worker.  Then every block of whole quads takes this path (all
// but perhaps the array's last block); any other block goes quad by quad or element by element and forms its
// means once for the maximum and once for the compression.
// Calls f(first quad, G) for the groups 0, 1, ... of G quads each, in order.
template <int G, typename F, int... I>
__device__ __forceinline__ void encode_groups(F &f, std::integer_sequence<int, I...>)
{
    ((f(std::integral_constant<int, I * G>{}, std::integral_constant<int, G>{}), __builtin_amdgcn_sched_barrier(0)), ...);
}

constexpr int kLongWaves = 8;                  // wavefronts per block in k_avg_long
constexpr int kLongTeam = kLongWaves * kWave;  // its threads
constexpr int kLongSlots = 2 * kLongWaves;     // LDS words for the maxima (two phases)

template <int QL, int NB, int NT, int KT>
__global__ __launch_bounds__(kLongTeam) void k_avg_long(const uint32_t *__restrict__ tab, WorkerPtrs p, int K_rt,
                                                 const float *__restrict__ local, size_t n, size_t B, size_t nb,
                                                 uint32_t n_teams, uint32_t aligned, float *__restrict__ scales_out,
                                                 uint8_t *__restrict__ codes_out)
{
    static_assert(NB >= 2, "at least two sets of code words");
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t dyn_lds[];  // kLongSlots words for the maxima, then the bucket table
    constexpr int Q = QL;
    const int K = KT > 0 ? KT : K_rt;  // KT > 0: the number of workers is known at compile time
    const int terms = K + (local ? 1 : 0);
    const float fk = (float)terms;
    const bool pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    const float rk = 1.0f / fk;
    auto mean_of = [&](float acc) { return pow2 ? acc * rk : acc / fk; };
    const uint32_t lane = threadIdx.x & 63, wave = wave_in_wg(), tl = threadIdx.x;
    const uint32_t lane4 = lane * 4;
    uint32_t *slots = dyn_lds;
    uint32_t phase = 0;
    load_lut(tab, lut);
    const Search sr = load_bucket_table(tab, dyn_lds + kLongSlots, kLongTeam);
    __syncthreads();
    // Maximum over the workgroup of the wave maxima m, through LDS; one barrier per call.
    auto team_max = [&](uint32_t m) {
        if (lane == 0) slots[phase * kLongWaves + wave] = m;
        __syncthreads();
        const uint32_t *sp = slots + phase * kLongWaves;
        uint32_t a = sp[0];
#pragma unroll
        for (int i = 1; i < kLongWaves; ++i) a = a > sp[i] ? a : sp[i];
        phase ^= 1;  // the other half of slots next time
        return (uint32_t)__builtin_amdgcn_readfirstlane((int)a);
    };
    auto length_of = [&](size_t blk) { return (uint32_t)(n - blk * B < B ? n - blk * B : B); };
    // Blocks 0 .. n_stream - 1 take the register path: all of them when the array's last block is whole quads.
    const uint32_t last_len = length_of(nb - 1);
    const size_t n_stream = !aligned ? 0 : ((last_len >= 4 && (last_len & 3) == 0) ? nb : nb - 1);
    if (blockIdx.x < n_stream) {
        const int Kp = (K + NB - 1) / NB * NB;  // places per block
        uint32_t w[NB][Q];                      // the sets of code words
        float scv[NB];                          // and the scale that belongs to each
        // Requests place `place` of block b: scale and code words of worker `place`, or of the last worker again.
        auto request = [&](uint32_t(&ww)[Q], float &sc, size_t b, int place) {
            const int worker = place < K ? place : K - 1;
            const uint32_t last = (length_of(b) >> 2) - 1;
            sc = ldg<0>(p.scales[worker] + b);
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[worker] + b * B);
#pragma unroll
            for (int j = 0; j < Q; ++j) {
                const uint32_t i = j * kLongTeam + tl;
                ww[j] = ldg_at<NT>(c4, i < last ? i : last);
            }
        };
        // (one set after the other, as in the loop below: the waits there are counted for the worse of the two orders)
#pragma unroll
        for (int i = 0; i < NB - 1; ++i) {
            request(w[i], scv[i], blockIdx.x, i);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (size_t blk = blockIdx.x; blk < n_stream; blk += n_teams) {
            const size_t start = blk * B;
            const size_t next = blk + n_teams < n_stream ? blk + n_teams : blk;  // after the last block: this one again
            const uint32_t nq = length_of(blk) >> 2, last = nq - 1;
            v4f acc[Q];
            if (local) {  // not requested ahead: the sums are still in use when the code words of this block set out
                const v4f *l4 = reinterpret_cast<const v4f *>(local + start);
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    const uint32_t i = j * kLongTeam + tl;
                    acc[j] = ldg_at<NT>(l4, i < last ? i : last);
                }
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
            auto add_w = [&](const uint32_t(&ww)[Q], float sk) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    acc[j].x = acc[j].x + lut_at<0>(lut, ww[j], lane4) * sk;
                    acc[j].y = acc[j].y + lut_at<1>(lut, ww[j], lane4) * sk;
                    acc[j].z = acc[j].z + lut_at<2>(lut, ww[j], lane4) * sk;
                    acc[j].w = acc[j].w + lut_at<3>(lut, ww[j], lane4) * sk;
                }
                // pin the sums here, or the compiler defers them and holds the products of several workers
#pragma unroll
                for (int j = 0; j < Q; ++j) asm volatile("" : "+v"(acc[j].x), "+v"(acc[j].y), "+v"(acc[j].z), "+v"(acc[j].w));
            };
            // One round: NB steps, each requesting the place NB - 1 ahead (in the next block once this block's places
            // are all requested) and adding the oldest set.
            bool in_range = !pow2 && !local;  // the sums are going to be divided and are 0 or where divide_by_count holds
            auto round = [&](int k) {
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int ahead = k + i + NB - 1;
                    const bool wraps = ahead >= Kp;
                    request(w[(i + NB - 1) % NB], scv[(i + NB - 1) % NB], wraps ? next : blk, wraps ? ahead - Kp : ahead);
                    // the scale is the same in every lane: to a scalar register, and its range test on the scalar unit
                    const uint32_t sb = k + i < K ? (uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(scv[i])) : 0u;
                    if (in_range) in_range = scale_keeps_sums_in_range(sb);
                    add_w(w[i], u2f(sb));
                }
            };
            if constexpr (KT > 0) {
#pragma unroll
                for (int k = 0; k < (KT + NB - 1) / NB * NB; k += NB) round(k);
            } else {
                for (int k = 0; k < Kp; k += NB) round(k);
            }
            float pre;  // what the sums still have to be multiplied by to be the means: 1 here (registers)
            const float fm = means_for_compression<Q, false>(acc, pow2, rk, fk, &pre, in_range);
            const float s = u2f(team_max(wave_max_u32(f2u(fm))));
            if (tl == 0) scales_out[blk] = s;
            const float d = s == 0.0f ? 1.0f : s;
            const float r = 1.0f / d;
            const bool recip = reciprocal_ok(d);
            uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out + start);
            // quads whose table lookups are issued together: four, and what is left of Q after the groups of four
            auto encode_group = [&](auto first, auto count) {
                constexpr int g = decltype(first)::value, G = decltype(count)::value;
                v4f vv[G];
                uint32_t cw[G];
#pragma unroll
                for (int j = 0; j < G; ++j) vv[j] = acc[g + j];
                encode_quads<true, G>(sr, vv, pre, d, r, recip, cw);
#pragma unroll
                for (int j = 0; j < G; ++j)
                    if ((g + j) * kLongTeam + tl < nq) stg<1>(c4 + (g + j) * kLongTeam + tl, cw[j]);
            };
            // groups of four quads, of two where a lane holds seven or eight (the sums of a group are all live at
            // once; with larger groups two workgroups no longer fit a compute unit's registers), one group after the other
            constexpr int G = Q >= 7 ? 2 : 4;
            encode_groups<G>(encode_group, std::make_integer_sequence<int, Q / G>{});
            if constexpr (Q % G != 0)
                encode_group(std::integral_constant<int, Q / G * G>{}, std::integral_constant<int, Q % G>{});
        }
    }
    // The blocks that are not on the register path: all of them without `aligned`, else at most the array's last one.
    const size_t slow_first = aligned ? nb - 1 : 0;
    for (size_t blk = slow_first + (blockIdx.x + n_teams - slow_first % n_teams) % n_teams; blk < nb; blk += n_teams) {
        if (blk < n_stream) continue;
        const size_t start = blk * B;
        const uint32_t len = length_of(blk);
        const bool quads_ok = [&] {
            bool ok = ((uintptr_t)(codes_out + start) & 3) == 0;
            for (int k = 0; k < K; ++k) ok = ok && (((uintptr_t)(p.codes[k] + start) & 3) == 0);
            if (local) ok = ok && (((uintptr_t)(local + start) & 15) == 0);
            return ok;
        }();
        const uint32_t nq = quads_ok ? len >> 2 : 0;
        const uint32_t done = nq << 2;
        auto mean_at = [&](uint32_t i) {
            float a = 0.0f;
            if (local) a = a + local[start + i];
            for (int k = 0; k < K; ++k) a = a + lut_code(lut, p.codes[k][start + i], lane4) * p.scales[k][blk];
            return mean_of(a);
        };
        auto mean_quad = [&](uint32_t q) {
            v4f a = {0.0f, 0.0f, 0.0f, 0.0f};
            if (local) {
                const v4f l = ldg<NT>(reinterpret_cast<const v4f *>(local + start) + q);
                a.x = a.x + l.x;
                a.y = a.y + l.y;
                a.z = a.z + l.z;
                a.w = a.w + l.w;
            }
            for (int k = 0; k < K; ++k) {
                const uint32_t ww = ldg<NT>(reinterpret_cast<const uint32_t *>(p.codes[k] + start) + q);
                const float sk = p.scales[k][blk];
                a.x = a.x + lut_at<0>(lut, ww, lane4) * sk;
                a.y = a.y + lut_at<1>(lut, ww, lane4) * sk;
                a.z = a.z + lut_at<2>(lut, ww, lane4) * sk;
                a.w = a.w + lut_at<3>(lut, ww, lane4) * sk;
            }
            a.x = mean_of(a.x);
            a.y = mean_of(a.y);
            a.z = mean_of(a.z);
            a.w = mean_of(a.w);
            return a;
        };
        float fm = 0.0f;
        for (uint32_t q = tl; q < nq; q += kLongTeam) fm = max4_abs(mean_quad(q), fm);
        uint32_t m = f2u(fm);
        for (uint32_t i = done + tl; i < len; i += kLongTeam) {
            const uint32_t a = abs_bits(mean_at(i));
            m = m > a ? m : a;
        }
        const float s = u2f(team_max(wave_max_u32(m)));
        if (tl == 0) scales_out[blk] = s;
        const float d = s == 0.0f ? 1.0f : s;
        const float r = 1.0f / d;
        const bool recip = reciprocal_ok(d);
        uint32_t *c4 = reinterpret_cast<uint32_t *>(codes_out + start);
        for (uint32_t q = tl; q < nq; q += kLongTeam) stg<1>(c4 + q, encode_quad<true>(sr, mean_quad(q), d, r, recip));
        for (uint32_t i = done + tl; i < len; i += kLongTeam)
            codes_out[start + i] = (uint8_t)encode_one<true>(sr, mean_at(i), d, r, recip);
    }
}

// The same average-then-compress round for up to eight workers (K fixed at compile time) at full speed.  A team of W
// wavefronts (four unless the blocks are shorter) owns a unit of W x 1024 elements (one scale block): every lane
// holds four quads of running sums and K x 4 code words.  The code words are one register set that is refilled
// in place: as soon as worker k's words of the current unit have been decoded and added, the
// loads of worker k's words of the team's next unit are issued into the same registers, so
// loads are in flight all through the reduction to the block maximum (wave reduction, then one
// LDS exchange between the team's wavefronts) and the compression from the registers.
// TEAMS teams share a workgroup and its tables; the workgroup barrier that separates the
// exchange of the maxima from their use is executed by every wavefront the same number of
// times (`iters`), whether or not its team still has a unit.
// RAGGED = true (chosen by the host for blocks shorter than the unit): a unit of fewer whole aligned quads
// takes the register path as well.
// MULTI = true: more workers than KT, taken KT at a time in `passes` passes over the same registers; a
// place of the last pass that has no worker repeats worker K - 1 with scale 0 (the product is a zero, and
// adding a zero leaves a sum that started at +0 unchanged).  K is then a run-time value.
template <int KT, int NT, bool FASTDIV, int TEAMS, bool RAGGED, bool MULTI, int W>
struct AvgTeam {
    static_assert(W >= 1 && W <= kWavesPerWg, "a team is one to four wavefronts");
    static constexpr int Q = 4;               // quads per lane
    static constexpr int kTeam = W * kWave;   // threads per team
    static constexpr int kTeamUnit = Q * 4 * kTeam;  // elements per unit

    const WorkerPtrs &p;  // the kernel's argument itself: a copy would have to live in scratch memory to be indexed
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
    int K;              // number of workers: KT unless MULTI
    int passes;         // ceil(K / KT)

    struct Slot {
        Unit un;
        bool active, fast;
    };

    __device__ __forceinline__ explicit AvgTeam(const WorkerPtrs &workers) : p(workers) {}

    __device__ __forceinline__ float mean_of(float acc) const { return pow2 ? acc * rk : acc / fk; }

    // Element i of the unit, the slow way.
    __device__ __forceinline__ float mean_at(const Unit &un, uint32_t i) const
    {
        float a = 0.0f;
        if (local) a = a + local[un.start + i];
        if (MULTI) {
            for (int k = 0; k < K; ++k) a = a + lut_code(lut, p.codes[k][un.start + i], lane4) * p.scales[k][un.block];
        } else {
#pragma unroll
            for (int k = 0; k < KT; ++k) a = a + lut_code(lut, p.codes[k][un.start + i], lane4) * p.scales[k][un.block];
        }
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
        bool f = (RAGGED ? (sl.un.len >= 4 && (sl.un.len & 3) == 0) : sl.un.len == (uint32_t)kTeamUnit) &&
                 (((uintptr_t)(codes_out + sl.un.start) & 3) == 0);
        if (MULTI) {
            for (int k = 0; k < K; ++k) f = f && (((uintptr_t)(p.codes[k] + sl.un.start) & 3) == 0);
        } else {
#pragma unroll
            for (int k = 0; k < KT; ++k) f = f && (((uintptr_t)(p.codes[k] + sl.un.start) & 3) == 0);
        }
        if (local) f = f && (((uintptr_t)(local + sl.un.start) & 15) == 0);
        sl.fast = f;
    }

    // This lane's j-th quad of the unit; WHOLE promises a whole unit, otherwise a quad past the
    // end of a shorter unit becomes the unit's last one (an unconditional load of valid memory whose result
    // is not stored and cannot change the maximum).
    template <bool WHOLE>
    __device__ __forceinline__ uint32_t quad_of(const Slot &sl, int j) const
    {
        const uint32_t i = j * kTeam + tl;
        if (WHOLE || !RAGGED) return i;
        const uint32_t last = (sl.un.len >> 2) - 1;
        return i < last ? i : last;
    }

    // Code words of `worker` for unit sl into place k.
    template <bool WHOLE>
    __device__ __forceinline__ void load_worker(const Slot &sl, int k, int worker)
    {
        const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[worker] + sl.un.start);
#pragma unroll
        for (int j = 0; j < Q; ++j) w[k][j] = ldg_at<NT>(c4, quad_of<WHOLE>(sl, j));
    }

    __device__ __forceinline__ void load_all(const Slot &sl)
    {
        if (sl.fast) {
#pragma unroll
            for (int k = 0; k < KT; ++k) load_worker<false>(sl, k, k);
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
        float pre = 1.0f;  // what the sums still have to be multiplied by to be the means
        // whether the sums are 0 or where divide_by_count holds (see scale_keeps_sums_in_range); only asked for when
        // the sums are going to be divided
        bool in_range = !pow2 && !local;
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
          for (int pass = 0; pass < (MULTI ? passes : 1); ++pass) {
            const int base = pass * KT;
            const bool last_pass = !MULTI || pass + 1 == passes;
            float sc[KT];  // the scales of this pass's workers for this block, moved to scalar registers
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const bool empty = MULTI && !(base + k < K);
                const int worker = empty ? K - 1 : base + k;
                const float sv = p.scales[worker][sl.un.block];
                sc[k] = u2f((uint32_t)__builtin_amdgcn_readfirstlane((int)f2u(empty ? 0.0f : sv)));
            }
            if (in_range) {  // (never with a power-of-two number of terms: nothing of this on that path)
#pragma unroll
                for (int k = 0; k < KT; ++k) in_range = in_range && scale_keeps_sums_in_range(f2u(sc[k]));
            }
            // The table lookups run one worker ahead of the sums: worker k + 1's sixteen lookups are issued
            // before worker k's values are multiplied and added, so the LDS latency of one worker hides behind
            // the arithmetic of the one before.  The scheduling barriers keep that order.
            float lv[2][Q][4];
            auto lookup = [&](int k, float(&dst)[Q][4]) {
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    dst[j][0] = lut_at<0>(lut, w[k][j], lane4);
                    dst[j][1] = lut_at<1>(lut, w[k][j], lane4);
                    dst[j][2] = lut_at<2>(lut, w[k][j], lane4);
                    dst[j][3] = lut_at<3>(lut, w[k][j], lane4);
                }
            };
            lookup(0, lv[0]);
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                if (k + 1 < KT) lookup(k + 1, lv[(k + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < Q; ++j) {
                    acc[j].x = acc[j].x + lv[k & 1][j][0] * sc[k];
                    acc[j].y = acc[j].y + lv[k & 1][j][1] * sc[k];
                    acc[j].z = acc[j].z + lv[k & 1][j][2] * sc[k];
                    acc[j].w = acc[j].w + lv[k & 1][j][3] * sc[k];
                }
                // Pin the sums here.  Otherwise the compiler holds the products of several workers in
                // registers until the ordered sums get to them, which costs a wavefront per SIMD.
#pragma unroll
                for (int j = 0; j < Q; ++j) asm volatile("" : "+v"(acc[j].x), "+v"(acc[j].y), "+v"(acc[j].z), "+v"(acc[j].w));
                // refill in place (the lookups of this place are issued): the next pass's worker of this unit, or
                // after the last pass the next unit's worker k
                if (!last_pass) {
                    const int next_worker = base + KT + k < K ? base + KT + k : K - 1;
                    load_worker<STEADY>(sl, k, next_worker);
                } else if (STEADY || nx.fast) {
                    load_worker<STEADY>(nx, k, k);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
          }
            m = f2u(means_for_compression<Q>(acc, pow2, rk, fk, &pre, in_range));
        } else {
            if (sl.active) {
                for (uint32_t i = tl; i < sl.un.len; i += kTeam) {
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
        if constexpr (W == 4) {
            const uint32_t a = sp[0] > sp[1] ? sp[0] : sp[1], b = sp[2] > sp[3] ? sp[2] : sp[3];
            m = (uint32_t)__builtin_amdgcn_readfirstlane((int)(a > b ? a : b));
        } else {
            uint32_t a = sp[0];
#pragma unroll
            for (int i = 1; i < W; ++i) a = a > sp[i] ? a : sp[i];
            m = (uint32_t)__builtin_amdgcn_readfirstlane((int)a);
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
            uint32_t cw[Q];
            encode_quads<FASTDIV, Q>(sr, acc, pre, d, r, recip, cw);
#pragma unroll
            for (int j = 0; j < Q; ++j)
                if (STEADY || !RAGGED || j * kTeam + tl < (sl.un.len >> 2)) stg<1>(c4 + j * kTeam + tl, cw[j]);
        } else {
            for (uint32_t i = tl; i < sl.un.len; i += kTeam)
                codes_out[sl.un.start + i] = (uint8_t)encode_one<FASTDIV>(sr, mean_at(sl.un, i), d, r, recip);
        }
    }
};

template <int KT, int NT, bool FASTDIV, int TEAMS, bool REMAP, bool RAGGED, bool MULTI, int W = kWavesPerWg>
__global__ __launch_bounds__(kWave * W * TEAMS, W * TEAMS == 12 ? 3 : 4) void k_avg_team(const uint32_t *__restrict__ tab, WorkerPtrs p,
                                                            int K_rt, const float *__restrict__ local, size_t n, size_t B,
                                                            size_t nb,
                                                            size_t n_units, size_t n_teams, uint32_t iters, uint32_t steady,
                                                            float *__restrict__ scales_out, uint8_t *__restrict__ codes_out)
{
    __shared__ __align__(256) float lut[256 * kLutCopies];
    extern __shared__ uint32_t dyn_lds[];  // 2 phases x TEAMS x 4 maxima, then the bucket table
    constexpr int kSlots = 2 * TEAMS * kWavesPerWg;
    static_assert(W * TEAMS % 4 == 0, "whole wavefronts per SIMD");
    using Avg = AvgTeam<KT, NT, FASTDIV, TEAMS, RAGGED, MULTI, W>;
    Avg e(p);
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
    e.team = wave / W;
    e.wv = wave % W;
    e.tl = (W & (W - 1)) == 0 ? threadIdx.x & (W * kWave - 1) : threadIdx.x - e.team * (W * kWave);  // thread within the team
    e.phase = 0;
    e.K = MULTI ? K_rt : KT;
    e.passes = (e.K + KT - 1) / KT;
    const int terms = e.K + (local ? 1 : 0);
    e.fk = (float)terms;
    e.rk = 1.0f / e.fk;
    e.pow2 = (terms & (terms - 1)) == 0;  // then acc * (1 / terms) equals acc / terms exactly
    size_t u = (size_t)blockIdx.x * TEAMS + e.team;
    typename Avg::Slot a, b;
    e.open(u, a);
    e.load_all(a);  // the first loads are in flight while the tables are copied
    load_lut(tab, lut);
    {
        e.sr = load_bucket_table(tab, dyn_lds + kSlots, kWave * W * TEAMS);
        e.sr.marks = REMAP;  // known at compile time: no test for marked code bytes in the loop
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

}  // namespace
