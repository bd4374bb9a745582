// dq8 kernels and C ABI for gfx950 (MI355X).  See include/dq8.h for the contract.
//
// Work decomposition shared by every kernel: the array is cut into UNITS.  A unit is a run of
// at most U consecutive elements that lies inside one scale block, so one scale applies to the
// whole unit: unit u = (block b, chunk c) covers elements
// [b*B + c*U, min(b*B + (c+1)*U, (b+1)*B, n)).  A 64-lane wavefront (or, in the fused encoder,
// a team of four) owns a unit at a time and walks units with a grid-wide stride, so at any
// moment the whole chip streams through one narrow window of each array; the host sizes the
// grid so that every wavefront gets the same number of units and all of them are resident.
// U is Q * 256 (times four for a team), Q being the number of 128-bit accesses a lane keeps in
// flight; the host picks it per call: no longer than a block where units may be pieces of a block,
// the smallest power of two that holds a block (at most 4096) where a whole block has to be held.
//
// Inside a unit lane L owns elements 4*(64*it + L) .. +3: fp32 data moves as one 128-bit
// access per lane (1 KiB contiguous per wave instruction) and the matching four codes as one
// 32-bit access (256 B contiguous per instruction).  A unit of fewer whole aligned quads stays on
// that path (lanes past its end load its last quad and store nothing); units whose addresses are
// not aligned for it take quad or element loops with identical arithmetic.
// Every loop is software-pipelined: the loads of a wavefront's next unit are issued before
// the current one is processed.
//
// Files: dq8_device.hpp (access policies, reductions, unit geometry, code search, decode table),
// dq8_kernels_codec.hpp (absmax, encode, decode), dq8_kernels_avg.hpp (decode-and-average),
// dq8_kernels_avg_encode.hpp (average in registers, store and / or compress), dq8_kernels_stats.hpp
// (error statistics), dq8_kernels_small.hpp (blocks shorter than 256 elements), dq8_tables.cpp
// (host-side table construction); this file holds the launch logic and the C ABI.
//
// Built with -ffp-contract=off: the decode-and-average sum must round the product and the sum
// separately.  Divisions are the compiler's correctly rounded ones.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "dq8.h"
#include "dq8_internal.h"
#include "dq8_launch.hpp"
#include "dq8_plan.hpp"
#include "dq8_tables.hpp"

#include "dq8_device.hpp"
#include "dq8_kernels_avg.hpp"
#include "dq8_kernels_avg_encode.hpp"
#include "dq8_kernels_codec.hpp"
#include "dq8_kernels_small.hpp"
#include "dq8_kernels_segments.hpp"
#include "dq8_kernels_stats.hpp"

namespace {

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
    bool has_remap[kKinds] = {false, false, false, false};  // code bytes of the type can carry marks (fix_marked_codes)
    uint32_t search_words[kKinds] = {0, 0, 0, 0};  // LDS words of a type's bucket table
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
            st.has_remap[k] = t.has_marks;
            st.search_words[k] = t.n_bucket;
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
    int avg_flat = 1;       //   up to 8 workers, blocks of whole quads that are not a power-of-two number of units: units by position
    int avg_wide = 8;       //   9 to 12 workers: the unrolled kernel with this many wavefronts per compute unit (0: the chunk kernel)
    int avg_chunk_all = 0;  //   1: that kernel for K = 2, 4, 8 as well
    int avg_chunk_wpc = 8;  //   wavefronts per compute unit of the kernel that takes the workers four at a time
    int avg_lean_wpw = 4;
    int copy_nt = 1;
    int fastdiv = 1;     // reciprocal multiply with exact fallback near thresholds
    int enc_wpb = 4;     // wavefronts per unit in the encoder: 1 or 4
    int enc_wpc = 24;    // encoder wavefronts per compute unit (general kernel)
    int enc_long = 1;    // blocks of 4097 .. 16384 elements: held by a team (0: absmax pass + encode pass, 2: general kernel only)
    int enc_wpc8 = 8;    //   wavefronts per compute unit with 8 quads per lane (measured: 8: 55, 12: 57, 16: 57 us at block 8192),
    int enc_wave_min = 8;   // blocks of this many
    int enc_wave = 1024;    //   up to this many elements: the wave-per-block kernel whose loads are a block ahead (0: off;
                            //   block 200: 114 -> 63 us, 600: 75 -> 56, 1000: 65 -> 57, 1024: 60 -> 54, 100: 202 -> 101)
    int enc_wave_wpc = 32;  //   its wavefronts per compute unit with 1 to 4 quads per lane,
    int enc_wave_wpc8 = 16; //   and with 8
    int enc_mid = 1536;  // blocks longer than this, up to 3072 elements: the same kernel (0: off; measured 1500: 62 -> 63 us,
                         //   2000: 60 -> 58, 2048: 57.5 -> 55, 3000: 62 -> 57.5, 3072: 58 -> 55, 4000: 56 -> 58)
    int enc_wpc4 = 16;   //   its wavefronts per compute unit with 2 or 3 quads per lane (8: 72, 16: 55, 24: 55, 32: 56 us at 2048)
    int enc_wpc6 = 12;   //   6 (12: 59, 20: 62 us at block 5000)
    int enc_wpc12 = 12;  //   and 12 (12: 56, 8: 57, 16: 57-59 us at block 9216 and 12288)
    int enc_wpc16 = 8;   //   16 (8: 57, 4: 64 us at block 16384),
    int enc_lean = 1;    // whole aligned 4096-element blocks go to the kernel without slow paths in its loop,
    int enc_lean_wpc = 8;  //   which keeps its loads in flight with this many wavefronts per compute unit
    int enc_fill = 1;    //   and puts a team on every resident slot, even if some then get one block fewer
    int amax_q = 16;     // absmax: quads per lane in flight (unit = 256 q elements)
    int amax_waste = 1;  //   smaller units for blocks whose last unit would be mostly empty
    int amax_wpc = 3;    //   wavefronts per compute unit: 3 measured best (36.2 us against 37.5 with 4 on 61 M elements)
    int dec_flat = 1;    // decode: units by position for blocks that are not whole units (0: off, 2: for every block length)
    int dec_q = 16;      // decode: code words per lane in flight
    int dec_wpc = 4;
    int dec_wpw = 4;     // decode: wavefronts per workgroup (they share one table in LDS)
    int avg_q = 2;       // decode-and-average: code words per lane and worker in flight
    int avg_wpc = 32;
    int avg_wpw = 16;
    int blk_wpw = 8;     // register-resident average: wavefronts per workgroup (two workgroups per compute unit)
    int avg_team = 1;    // average-then-compress with up to 8 workers: the team kernel (0: the wave-per-block kernel)
    int avg_steady = 1;  //   unconditional steady-state iterations when the buffers are aligned
    int avg_teams = 0;   //   teams per workgroup: 2, 3 or 4 (0: by the number of workers)
    int avg_teams4_upto = 6;  //   four teams for up to this many workers (K = 3: 79 -> 69 us, K = 6: 94 -> 92 us), three beyond (K = 8: 105 against 120 us)
    int avg_wgpc = 1;    //   workgroups per compute unit (2 only with 2 teams)
    int copy_q = 2;
    int copy_wpc = 8;
};
// The shipped library has fixed launch shapes: nothing mutable is shared between calls, so calls from several
// threads need no lock.  A build with -DDQ8_TUNABLE (experiments only) makes them changeable through
// dq8_internal_tune(), which is not synchronised with calls in flight on other threads.
#ifdef DQ8_TUNABLE
Tuning g_tune;
#else
const Tuning g_tune{};
#endif

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

// DQ8_DEBUG=1 in the environment (read once, at the first launch): every launch is followed by a wait for the
// stream and a check of the error state, so that a failing kernel is reported by the call that launched it.
bool debug_sync()
{
    static const bool on = [] {
        const char *v = std::getenv("DQ8_DEBUG");
        return v && v[0] != '\0' && std::strcmp(v, "0") != 0;
    }();
    return on;
}

int after_launch(const char *what, hipStream_t stream)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DQ8_ERR_DEVICE, "launch of %s failed: %s", what, hipGetErrorString(e));
    if (debug_sync()) {
        e = hipStreamSynchronize(stream);
        if (e == hipSuccess) e = hipGetLastError();
        if (e != hipSuccess) return fail(DQ8_ERR_DEVICE, "%s failed on the device: %s", what, hipGetErrorString(e));
    }
    return DQ8_OK;
}

// ---- blocks of 4 .. 128 elements (powers of two): kernels that pack many blocks into a wavefront's unit

#define DQ8_SMALL_G(lanes, CALL) \
    switch (lanes) {             \
    case 1: CALL(1); break;      \
    case 2: CALL(2); break;      \
    case 4: CALL(4); break;      \
    case 8: CALL(8); break;      \
    case 16: CALL(16); break;    \
    default: CALL(32); break;    \
    }
#define DQ8_SMALL_G256(lanes, CALL) \
    if (lanes == 64) {              \
        CALL(64);                   \
    } else if (lanes == 128) {      \
        CALL(128);                  \
    } else if (lanes == 256) {      \
        CALL(256);                  \
    } else {                        \
        DQ8_SMALL_G(lanes, CALL)    \
    }

// Each of these launches the short-block kernel on the leading whole units when the block length and the
// alignment allow it and returns in *done the number of elements covered (0: nothing was launched); the caller
// hands the rest, which starts on a block boundary, to the general kernels.
int small_absmax(const DeviceState &st, const float *x, size_t n, size_t block_len, float *scales, hipStream_t stream,
                 size_t *done)
{
    *done = 0;
    const int lanes = small_block_lanes(n, block_len);
    if (!lanes || ((uintptr_t)x & 15)) return DQ8_OK;
    const SmallPlan p = make_small_plan(n, st.cus, 32, kWavesPerWg);
    if (!p.n_units) return DQ8_OK;
#define DQ8_CALL(G) hipLaunchKernelGGL((k_small_absmax<kSmallQ, G>), dim3(p.grid), dim3(kWg), 0, stream, x, p.n_units, p.n_waves, scales)
    DQ8_SMALL_G(lanes, DQ8_CALL)
#undef DQ8_CALL
    *done = p.done;
    return after_launch("k_small_absmax", stream);
}

int small_encode(const DeviceState &st, int kind, const float *x, size_t n, size_t block_len, float *scales, uint8_t *codes,
                 bool given, hipStream_t stream, size_t *done)
{
    *done = 0;
    const int lanes = small_block_lanes(n, block_len, 512);
    if (!lanes || ((uintptr_t)x & 15) || ((uintptr_t)codes & 3)) return DQ8_OK;
    const SmallPlan p = make_small_plan(n, st.cus, 32, kWavesPerWg);
    if (!p.n_units) return DQ8_OK;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = (size_t)st.search_words[kind] * sizeof(uint32_t);
#define DQ8_CALL(G)                                                                                                      \
    if (given)                                                                                                           \
        hipLaunchKernelGGL((k_small_encode<kSmallQ, G, true>), dim3(p.grid), dim3(kWg), lds, stream, tab, x, p.n_units,   \
                           p.n_waves, scales, codes);                                                                    \
    else                                                                                                                 \
        hipLaunchKernelGGL((k_small_encode<kSmallQ, G, false>), dim3(p.grid), dim3(kWg), lds, stream, tab, x, p.n_units,  \
                           p.n_waves, scales, codes)
    DQ8_SMALL_G256(lanes, DQ8_CALL)
#undef DQ8_CALL
    *done = p.done;
    return after_launch("k_small_encode", stream);
}

int small_decode(const DeviceState &st, int kind, const uint8_t *codes, const float *scales, size_t n, size_t block_len,
                 float *out, hipStream_t stream, size_t *done)
{
    *done = 0;
    const int lanes = small_block_lanes(n, block_len);
    if (!lanes || ((uintptr_t)out & 15) || ((uintptr_t)codes & 3)) return DQ8_OK;
    const SmallPlan p = make_small_plan(n, st.cus, 32, 16);
    if (!p.n_units) return DQ8_OK;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
#define DQ8_CALL(G) \
    hipLaunchKernelGGL((k_small_decode<kSmallQ, G, 16>), dim3(p.grid), dim3(kWave * 16), 0, stream, tab, codes, scales, p.n_units, p.n_waves, out)
    DQ8_SMALL_G(lanes, DQ8_CALL)
#undef DQ8_CALL
    *done = p.done;
    return after_launch("k_small_decode", stream);
}

int small_avg(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n, size_t block_len,
              float *out, hipStream_t stream, size_t *done)
{
    *done = 0;
    const int lanes = small_block_lanes(n, block_len);
    bool ok = lanes != 0 && ((uintptr_t)out & 15) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) ok = ok && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (!ok) return DQ8_OK;
    const SmallPlan p = make_small_plan(n, st.cus, 32, 16);
    if (!p.n_units) return DQ8_OK;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
#define DQ8_CALL(G) \
    hipLaunchKernelGGL((k_small_avg<kSmallQ, G, 16>), dim3(p.grid), dim3(kWave * 16), 0, stream, tab, wp, K, local, p.n_units, p.n_waves, out)
    DQ8_SMALL_G(lanes, DQ8_CALL)
#undef DQ8_CALL
    *done = p.done;
    return after_launch("k_small_avg", stream);
}

int small_avg_encode(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                     size_t block_len, float *scales_out, uint8_t *codes_out, hipStream_t stream, size_t *done)
{
    *done = 0;
    const int lanes = small_block_lanes(n, block_len, kSmallUnit);
    bool ok = lanes != 0 && ((uintptr_t)codes_out & 3) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) ok = ok && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (!ok) return DQ8_OK;
    const SmallPlan p = make_small_plan(n, st.cus, 32, 16);
    if (!p.n_units) return DQ8_OK;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = (size_t)st.search_words[kind] * sizeof(uint32_t);
#define DQ8_CALL(G)                                                                                                       \
    hipLaunchKernelGGL((k_small_avg_encode<kSmallQ, G, 16>), dim3(p.grid), dim3(kWave * 16), lds, stream, tab, wp, K, local, \
                       p.n_units, p.n_waves, scales_out, codes_out)
    DQ8_SMALL_G256(lanes, DQ8_CALL)
#undef DQ8_CALL
    *done = p.done;
    return after_launch("k_small_avg_encode", stream);
}

// The worker pointers advanced by `done` elements (`done` a multiple of the block length).
WorkerPtrs advance_workers(const WorkerPtrs &wp, int K, size_t done, size_t block_len)
{
    WorkerPtrs r = wp;
    for (int k = 0; k < K; ++k) {
        r.codes[k] = wp.codes[k] + done;
        r.scales[k] = wp.scales[k] + done / block_len;
    }
    return r;
}

int launch_absmax(const DeviceState &st, const float *x, size_t n, size_t block, float *scales, hipStream_t stream)
{
    const size_t Bq = block_length(n, block);
    size_t done = 0;
    int rc0 = small_absmax(st, x, n, Bq, scales, stream, &done);
    if (rc0 || done == n) return rc0;
    x += done;  // the rest starts on a block boundary
    scales += done / Bq;
    n -= done;
    // Units no longer than a block (so that whole blocks are whole units when the block is a power of two),
    // and the more wavefronts per compute unit the smaller the unit: the bytes in flight stay the same.
    int q = (g_tune.amax_q == 1 || g_tune.amax_q == 2 || g_tune.amax_q == 8 || g_tune.amax_q == 16) ? g_tune.amax_q : 4;
    // three wavefronts per compute unit are the best when every unit is a whole full-size one; four otherwise
    // (smaller units, or blocks that end inside units)
    const size_t full_unit = (size_t)q * 4 * kWave;
    int wpc = (Bq >= n || Bq % full_unit == 0) ? g_tune.amax_wpc : 4;
    fit_unit_to_block(Bq, &q, &wpc);
    if (g_tune.amax_waste && Bq < n) {
        // A block that is not whole units ends in a short unit, whose lanes repeat loads.  Smaller units (down to
        // 1024 elements) when they cut what the units of a block cover beyond the block by more than 5 %.
        auto covered = [&](int quads) {
            const size_t unit = (size_t)quads * 4 * kWave;
            return (Bq + unit - 1) / unit * unit;
        };
        int best = q, best_wpc = wpc;
        for (int qq = q / 2, ww = wpc * 2; qq >= 4; qq /= 2, ww *= 2)
            if (covered(qq) * 100 < covered(best) * 95) {
                best = qq;
                best_wpc = ww > 32 ? 32 : ww;
            }
        q = best;
        wpc = best_wpc;
    }
    Plan p = make_plan(n, block, st.cus, wpc, 1, kWavesPerWg, (size_t)q * 4 * kWave);
    size_t per_wave = 0;
    if (p.upb > 1) {
        unsigned g = (unsigned)((p.nb + 255) / 256);
        hipLaunchKernelGGL(k_fill_zero, dim3(g), dim3(256), 0, stream, scales, p.nb);
        int rc = after_launch("k_fill_zero", stream);
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
    return after_launch("k_absmax", stream);
}

int launch_encode(const DeviceState &st, int kind, const float *x, size_t n, size_t block, float *scales, uint8_t *codes,
                  bool fused, hipStream_t stream)
{
    // Unit = the smallest power of two that holds a block, from 256 elements up to 4096 (scales given) or 16384
    // (scales computed here).  4096 and more: a team of four wavefronts per unit with 4, 8 or 16 quads per lane.
    // Smaller: one wavefront per unit (1, 2, 4 or 8 quads per lane) and every wavefront slot of the compute
    // units in use.
    const size_t Bq = block_length(n, block);
    const size_t unit = encode_unit(Bq, fused);
    const bool small = unit < (size_t)kUnit;
    const int wpb = small ? 1 : ((g_tune.enc_wpb == 4 || unit > (size_t)kUnit) ? 4 : 1);
    const int ql = (int)(unit / (size_t)(4 * kWave * wpb));
    // resident wavefronts per compute unit: what the registers of the longer units leave room for
    const int wpc = small ? 32 : (unit == 8192 ? 16 : (unit == 16384 ? 8 : g_tune.enc_wpc));
    Plan p = make_plan(n, block, st.cus, wpc, wpb, kWavesPerWg, unit);
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
        return after_launch("k_encode_full", stream);
    }
    // Blocks of 4097 .. 16384 elements in whole quads, aligned buffers: the team holds a block in 8, 12 or 16
    // quads per lane.
    const size_t tail = n % p.B;
    // Blocks of up to 1024 elements in whole quads, aligned buffers: one wavefront per block with its loads
    // always a block ahead (blocks of 4 .. 128 elements that are powers of two went to the small kernels before).
    if (fused && g_tune.enc_wave && p.B >= (size_t)g_tune.enc_wave_min && p.B <= (size_t)g_tune.enc_wave && (p.B & 3) == 0 && (tail & 3) == 0 &&
        p.nb > 1 && p.nb < 0xFFFFFFFFull && ((uintptr_t)x & 15) == 0 && ((uintptr_t)codes & 3) == 0) {
        const uint32_t bq = (uint32_t)(p.B / 4), tail_q = (uint32_t)(tail / 4);
        const int wq = bq <= 64 ? 1 : (bq <= 128 ? 2 : (bq <= 256 ? 4 : 8));  // quads per lane
        const int ww = 16;                                                     // wavefronts per workgroup
        size_t waves = (size_t)st.cus * (size_t)(wq == 8 ? g_tune.enc_wave_wpc8 : g_tune.enc_wave_wpc);
        if (waves > p.nb) waves = p.nb;
        const unsigned grid = (unsigned)((waves + ww - 1) / ww);
        const uint32_t n_waves = grid * (uint32_t)ww;
        const size_t wlds = (size_t)st.search_words[kind] * sizeof(uint32_t);
#define DQ8_ENC_WAVE(QL)                                                                                              \
    if (st.has_remap[kind]) {                                                                                         \
        hipLaunchKernelGGL((k_encode_wave<QL, 1, 16, true>), dim3(grid), dim3(kWave * 16), wlds, stream, tab, x,      \
                           (uint32_t)p.nb, n_waves, bq, tail_q, scales, codes);                                       \
    } else {                                                                                                          \
        hipLaunchKernelGGL((k_encode_wave<QL, 1, 16, false>), dim3(grid), dim3(kWave * 16), wlds, stream, tab, x,     \
                           (uint32_t)p.nb, n_waves, bq, tail_q, scales, codes);                                       \
    }
        switch (wq) {
        case 1: DQ8_ENC_WAVE(1) break;
        case 2: DQ8_ENC_WAVE(2) break;
        case 4: DQ8_ENC_WAVE(4) break;
        default: DQ8_ENC_WAVE(8) break;
        }
#undef DQ8_ENC_WAVE
        return after_launch("k_encode_wave", stream);
    }
    const bool long_block = unit > (size_t)kUnit;
    // blocks of 1537 .. 3072 elements too: 2 or 3 quads per lane (2 to 7 % faster than a wavefront per block there)
    const bool mid_block = g_tune.enc_mid && p.B > (size_t)g_tune.enc_mid && p.B <= 3072;
    if (fused && g_tune.enc_long == 1 && (long_block || mid_block) && (p.B & 3) == 0 &&
        (tail & 3) == 0 && p.nb < 0xFFFFFFFFull && ((uintptr_t)x & 15) == 0 && ((uintptr_t)codes & 3) == 0) {
        const uint32_t bq = (uint32_t)(p.B / 4), tail_q = (uint32_t)(tail / 4);
        const int qpl = bq <= 512 ? 2 : (bq <= 768 ? 3 : (bq <= 1536 ? 6 : (bq <= 2048 ? 8 : (bq <= 3072 ? 12 : 16))));  // quads per lane
        const int lwpc = qpl <= 3 ? g_tune.enc_wpc4 : (qpl == 6 ? g_tune.enc_wpc6 : (qpl == 8 ? g_tune.enc_wpc8 : (qpl == 12 ? g_tune.enc_wpc12 : g_tune.enc_wpc16)));
        size_t teams = (size_t)st.cus * (size_t)lwpc / 4;
        if (teams > p.nb) teams = p.nb;
#define DQ8_ENC_LONG(QPL)                                                                                             \
    if (st.has_remap[kind]) {                                                                                         \
        hipLaunchKernelGGL((k_encode_long<QPL, 1, true>), dim3((unsigned)teams), dim3(kWg), lds, stream, tab, x,      \
                           (uint32_t)p.nb, (uint32_t)teams, bq, tail_q, scales, codes);                               \
    } else {                                                                                                          \
        hipLaunchKernelGGL((k_encode_long<QPL, 1, false>), dim3((unsigned)teams), dim3(kWg), lds, stream, tab, x,     \
                           (uint32_t)p.nb, (uint32_t)teams, bq, tail_q, scales, codes);                               \
    }
        if (qpl == 2) {
            DQ8_ENC_LONG(2)
        } else if (qpl == 3) {
            DQ8_ENC_LONG(3)
        } else if (qpl == 6) {
            DQ8_ENC_LONG(6)
        } else if (qpl == 8) {
            DQ8_ENC_LONG(8)
        } else if (qpl == 12) {
            DQ8_ENC_LONG(12)
        } else {
            DQ8_ENC_LONG(16)
        }
#undef DQ8_ENC_LONG
        return after_launch("k_encode_long", stream);
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
    if (wpb == 4 && ql == 8) {
        DQ8_ENC(4, 8, true, true);
    } else if (wpb == 4 && ql == 16) {
        DQ8_ENC(4, 16, true, true);
    } else if (wpb == 4) {
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
    return after_launch("k_encode", stream);
}

// Error statistics of compress-then-decompress into stats[4 nb] (and means[2] when not NULL).
int launch_error_stats(const DeviceState &st, int kind, const float *x, size_t n, size_t block, const float *scales,
                       double *stats, double *means, hipStream_t stream)
{
    constexpr int Q = 4;
    constexpr int kWavesPerCu = 2 * kStatsWaves;  // two workgroups
    Plan p = make_plan(n, block, st.cus, kWavesPerCu, 1, kStatsWaves, (size_t)Q * 4 * kWave);
    const size_t n_waves = (size_t)p.grid * kStatsWaves;
    // Wavefronts own whole blocks when there is at least one block for each of them and a block is at most 64 units
    // (then no wavefront's share of the work is far from the average); otherwise they share blocks through atomics
    // on zeroed rows.
    const size_t all_waves = (size_t)st.cus * kWavesPerCu;
    const bool own = p.upb <= 64 && p.nb >= all_waves;
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const size_t lds = (size_t)st.search_words[kind] * sizeof(uint32_t);
    int rc;
    if (own) {
        const unsigned grid = (unsigned)(all_waves / kStatsWaves);
        hipLaunchKernelGGL((k_error_stats<Q, true>), dim3(grid), dim3(kStatsWg), lds, stream, tab, x, n, p.B, p.nb, p.upb,
                           p.n_units, (size_t)0, all_waves, scales, stats);
        rc = after_launch("k_error_stats", stream);
    } else {
        const size_t zero_words = 8 * p.nb;  // 4 binary64 zeros per block
        hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, stream,
                           reinterpret_cast<float *>(stats), zero_words);
        rc = after_launch("k_fill_zero", stream);
        if (rc) return rc;
        const size_t per_wave = (p.n_units + n_waves - 1) / n_waves;
        hipLaunchKernelGGL((k_error_stats<Q, false>), dim3(p.grid), dim3(kStatsWg), lds, stream, tab, x, n, p.B, p.nb, p.upb,
                           p.n_units, per_wave, n_waves, scales, stats);
        rc = after_launch("k_error_stats", stream);
    }
    if (rc || !means) return rc;
    hipLaunchKernelGGL(k_error_means, dim3(1), dim3(kMeansThreads), 0, stream, stats, p.nb, n, means);
    return after_launch("k_error_means", stream);
}

int launch_decode(const DeviceState &st, int kind, const uint8_t *codes, const float *scales, size_t n, size_t block,
                  float *out, hipStream_t stream)
{
    // Units no longer than a block, and the smaller the unit the more wavefronts per compute unit (the bytes
    // in flight stay the same); 16 wavefronts share a workgroup's 64 KiB table when there are that many.
    const size_t Bq = block_length(n, block);
    int q = (g_tune.dec_q == 1 || g_tune.dec_q == 2 || g_tune.dec_q == 4 || g_tune.dec_q == 8) ? g_tune.dec_q : 16;
    int wpc = g_tune.dec_wpc;
    fit_unit_to_block(Bq, &q, &wpc);
    const int wpw = q == 16 ? (g_tune.dec_wpw == 16 ? 16 : (g_tune.dec_wpw == 8 ? 8 : 4)) : (q == 8 ? 8 : 16);
    Plan p = make_plan(n, block, st.cus, wpc, 1, wpw, (size_t)q * 4 * kWave);
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    const bool ragged = p.nb > 1 && p.B % ((size_t)q * 4 * kWave) != 0;  // blocks end inside units
    // Blocks that do not consist of whole units (or, dec_flat == 2, any): units by position, not by block, with up
    // to eight blocks' scales per unit.  Needs blocks of whole quads and aligned buffers.
    const size_t bq = p.B / 4;
    // (also blocks of 2048 elements: 54 against 57 us with units of that length)
    if (g_tune.dec_flat && (ragged || g_tune.dec_flat == 2 || p.B == 2048) && p.nb > 1 && (p.B & 3) == 0 && bq >= 10 && bq < (1u << 28) &&
        ((uintptr_t)out & 15) == 0 && ((uintptr_t)codes & 3) == 0) {
        int fq = 16, fwpc = g_tune.dec_wpc;
        while ((size_t)fq * kWave > 7 * bq) {  // at most eight blocks per unit
            fq >>= 1;
            fwpc = fwpc * 2 > 32 ? 32 : fwpc * 2;
        }
        const bool four = (size_t)fq * kWave <= 3 * bq;  // at most four: fewer compares per quad
        const int fw = fq == 16 ? 4 : (fq == 8 ? 8 : 16);  // wavefronts per workgroup (they share the table)
        const uint64_t nq = n / 4, uq = (uint64_t)fq * kWave, n_units = (nq + uq - 1) / uq;
        uint64_t waves = (uint64_t)st.cus * (uint64_t)fwpc;
        if (waves > n_units) waves = n_units;
        if (waves < 1) waves = 1;
        const unsigned grid = (unsigned)((waves + fw - 1) / fw);
        const uint32_t n_waves = grid * (uint32_t)fw;
        const uint64_t step = (uint64_t)n_waves * uq;
#define DQ8_DEC_FLAT_N(Q, NS, WPW)                                                                                       \
    hipLaunchKernelGGL((k_decode_flat<Q, NS, 2, WPW>), dim3(grid), dim3(kWave * WPW), 0, stream, tab, codes, scales, nq, \
                       (uint32_t)(n & 3), (uint32_t)bq, (uint64_t)p.nb, n_units, n_waves, step / bq, (uint32_t)(step % bq), out)
#define DQ8_DEC_FLAT(Q, WPW)           \
    if (four) {                        \
        DQ8_DEC_FLAT_N(Q, 4, WPW);     \
    } else {                           \
        DQ8_DEC_FLAT_N(Q, 8, WPW);     \
    }
        switch (fq) {
        case 1: DQ8_DEC_FLAT(1, 16); break;
        case 2: DQ8_DEC_FLAT(2, 16); break;
        case 4: DQ8_DEC_FLAT(4, 16); break;
        case 8: DQ8_DEC_FLAT(8, 8); break;
        default: DQ8_DEC_FLAT(16, 4); break;
        }
#undef DQ8_DEC_FLAT
#undef DQ8_DEC_FLAT_N
        return after_launch("k_decode_flat", stream);
    }
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
    return after_launch("k_decode", stream);
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

// Whether a block of Bq <= 3072 elements goes to teams of one, two or three wavefronts: up to eight workers; a single
// worker only with three wavefronts (with one worker's code words in flight per team the sixteen wavefronts per compute
// unit of the wave-per-block kernels do better on the shorter blocks: 53 against 61 us at block 1000).
inline bool short_team_k(int K, size_t Bq) { return K >= (Bq > 2048 ? 1 : 2) && K <= 8; }

// Average-then-compress for blocks of up to 3072 elements: teams of W = 1, 2 or 3 wavefronts (dq8_avg_short.hip).
int launch_avg_short_team(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                          size_t block, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    return dq8::launch_avg_short_team_tu(st.cus, st.tables + (size_t)kind * kTableWords, st.search_words[kind], st.has_remap[kind],
                                         wp.codes, wp.scales, K, local, n, block, scales_out, codes_out, stream);
}

// Average-then-compress for up to 8 workers: teams of four wavefronts; two teams per workgroup and two
// workgroups per compute unit (128 registers per lane), or three teams in one workgroup per compute
// unit (170 registers per lane).
int launch_avg_team(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                    size_t block, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    const size_t Bq = block_length(n, block);
    if (Bq <= 3 * 1024 && short_team_k(K, Bq)) return launch_avg_short_team(st, kind, wp, K, local, n, block, scales_out, codes_out, stream);
    const bool ragged = Bq != (size_t)kUnit;  // shorter blocks: the variant whose register path takes short units
    const bool tuned_k = K == 2 || K == 4 || K == 8;  // the worker counts with a variant for 2 teams
    // Teams per workgroup: 3; 4 when each team has few code words in flight (up to `avg_teams4_upto` workers);
    // avg_teams overrides this where the variant exists.
    int teams = (K >= 1 && K <= g_tune.avg_teams4_upto && K <= 6) ? 4 : 3;
    if (g_tune.avg_teams == 3 || g_tune.avg_teams == 4) teams = g_tune.avg_teams;
    if (g_tune.avg_teams == 2 && tuned_k) teams = 2;
    if (ragged || K == 7 || K > 8) teams = 3;
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
#define DQ8_TEAM_M(KT, RM, T, RG, MU)                                                                                     \
    hipLaunchKernelGGL((k_avg_team<KT, 1, true, T, RM, RG, MU>), dim3(p.grid), dim3(kWg * T), lds, stream, tab, wp, K, local, \
                       n, p.B, p.nb, p.n_units, p.n_teams, iters, steady, scales_out, codes_out)
#define DQ8_TEAM(KT, RM, T, RG) DQ8_TEAM_M(KT, RM, T, RG, false)
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
    // K = 1, 3, 5, 6: three or four teams per workgroup; K = 7: three
#define DQ8_TEAM_34(KT, RM)                  \
    if (ragged) {                            \
        DQ8_TEAM(KT, RM, 3, true);           \
    } else if (teams == 4) {                 \
        DQ8_TEAM(KT, RM, 4, false);          \
    } else {                                 \
        DQ8_TEAM(KT, RM, 3, false);          \
    }
#define DQ8_TEAM_3(KT)                       \
    if (st.has_remap[kind]) {                \
        DQ8_TEAM_34(KT, true)                \
    } else {                                 \
        DQ8_TEAM_34(KT, false)               \
    }
#define DQ8_TEAM_7(KT)                       \
    if (st.has_remap[kind]) {                \
        if (ragged) {                        \
            DQ8_TEAM(KT, true, 3, true);     \
        } else {                             \
            DQ8_TEAM(KT, true, 3, false);    \
        }                                    \
    } else if (ragged) {                     \
        DQ8_TEAM(KT, false, 3, true);        \
    } else {                                 \
        DQ8_TEAM(KT, false, 3, false);       \
    }
    if (K > 8) {
        // more than 8 workers (whole 4096-blocks only): 5 to 8 at a time over the same registers, the count with the
        // fewest empty places in the last pass, the largest such
        int ch = 8;
        for (int c = 5, waste = DQ8_MAX_K; c <= 8; ++c) {
            const int w = (K + c - 1) / c * c - K;
            if (w <= waste) {
                waste = w;
                ch = c;
            }
        }
#define DQ8_TEAM_MULTI(KT)                           \
    if (st.has_remap[kind]) {                        \
        DQ8_TEAM_M(KT, true, 3, false, true);        \
    } else {                                         \
        DQ8_TEAM_M(KT, false, 3, false, true);       \
    }
        switch (ch) {
        case 5: DQ8_TEAM_MULTI(5) break;
        case 6: DQ8_TEAM_MULTI(6) break;
        case 7: DQ8_TEAM_MULTI(7) break;
        default: DQ8_TEAM_MULTI(8) break;
        }
#undef DQ8_TEAM_MULTI
        return after_launch("k_avg_team", stream);
    }
    switch (K) {
    case 1: DQ8_TEAM_3(1) break;
    case 2: DQ8_TEAM_RM(2) break;
    case 3: DQ8_TEAM_3(3) break;
    case 4: DQ8_TEAM_RM(4) break;
    case 5: DQ8_TEAM_3(5) break;
    case 6: DQ8_TEAM_3(6) break;
    case 7: DQ8_TEAM_7(7) break;
    default: DQ8_TEAM_RM(8) break;
    }
#undef DQ8_TEAM_7
#undef DQ8_TEAM_3
#undef DQ8_TEAM_34
#undef DQ8_TEAM_RM
#undef DQ8_TEAM_T
#undef DQ8_TEAM
#undef DQ8_TEAM_M
    return after_launch("k_avg_team", stream);
}

// Average-then-compress for blocks of 4097 .. kLongestHeldBlock elements: a workgroup per block (dq8_avg_long.hip).
int launch_avg_long(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                    size_t block, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    return dq8::launch_avg_long_tu(st.cus, st.tables + (size_t)kind * kTableWords, st.search_words[kind], wp.codes, wp.scales, K,
                                   local, n, block, scales_out, codes_out, stream);
}

int launch_avg_block(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                     size_t block, float *mean_out, float *scales_out, uint8_t *codes_out, hipStream_t stream)
{
    // Unit = the smallest power of two that holds a block, between 256 and 4096 elements.
    const size_t Bq = block_length(n, block);
    const size_t unit = holding_unit(Bq);
    // blocks that need a 4096-element unit with up to 8 workers, or exactly 4096 elements with more: the team kernel
    if (codes_out && !mean_out && K >= 1 && (K <= 8 || Bq == (size_t)kUnit) && g_tune.avg_team && unit == (size_t)kUnit)
        return launch_avg_team(st, kind, wp, K, local, n, block, scales_out, codes_out, stream);
    // blocks of 513 .. 2048 elements with a worker count that has kernels for shorter teams
    if (codes_out && !mean_out && g_tune.avg_team && Bq > 512 && Bq < n && short_team_k(K, Bq))
        return launch_avg_short_team(st, kind, wp, K, local, n, block, scales_out, codes_out, stream);
    const int ql = (int)(unit / (size_t)(4 * kWave));
    // whole 4096-element units with short ends need the 170 registers per lane that six wavefronts leave
    const bool ragged = Bq < n && Bq % unit != 0;  // blocks end inside units
    const int wpw = ql <= 4 ? 16 : ((ql == 16 && (ragged || g_tune.blk_wpw != 8)) ? 6 : 8);
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
    case 1: DQ8_BLK_R(1, 16) break;
    case 2: DQ8_BLK_R(2, 16) break;
    case 4: DQ8_BLK_R(4, 16) break;
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
    return after_launch("k_avg_block", stream);
}

// K-way decode-and-average (optional local term) of whole aligned units with a power-of-two number of them
// per block (or a single block): the kernels without slow paths in their loops, one unrolled for up to 8
// workers, one that takes any number of workers a chunk at a time.
// *launched = false (and nothing done) when the buffers do not qualify.
int launch_avg_full(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, const float *local, size_t n,
                    const Plan &p, float *out, hipStream_t stream, bool *launched)
{
    *launched = false;
    const int lq = g_tune.avg_lean_q == 4 ? 4 : 2;
    // wavefronts per workgroup (they share the 64 KiB decode table, two workgroups fit a compute unit): eight where
    // eight or more wavefronts per compute unit are wanted (up to 5 workers, see kWavesForK), else four
    const int lw_tuned = g_tune.avg_lean_wpw == 16 ? 16 : (g_tune.avg_lean_wpw == 8 ? 8 : 4);
    const int lw = (K >= 1 && K <= 5 && lw_tuned < 8) ? 8 : lw_tuned;
    const size_t U = (size_t)lq * 4 * kWave;
    const size_t upb_l = p.B / U;
    const bool by_shift = p.nb == 1 || (p.B % U == 0 && (upb_l & (upb_l - 1)) == 0);  // a unit's block is u >> shift
    // otherwise, for up to 8 workers: blocks of whole quads, no shorter than a unit (or exactly half a unit), two
    // blocks' scales per unit
    const size_t bq = p.B / 4;
    const bool flat_ok = !by_shift && g_tune.avg_flat && lq == 2 && (p.B & 3) == 0 && (bq >= U / 4 || bq * 2 == U / 4) &&
                         bq < 0x7FFFFFFFull && p.nb < 0xFFFFFFFFull;
    const bool flat = flat_ok && !g_tune.avg_chunk_all && K >= 1 && K <= 8;
    const bool flat_chunks = flat_ok && K > 8;  // more workers: the chunk kernel with the same geometry
    bool ok = by_shift || flat || flat_chunks;
    ok = ok && n / U >= 1 && n / U < 0x7FFFFFFFull && ((uintptr_t)out & 15) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) ok = ok && ((uintptr_t)wp.codes[k] & 3) == 0;
    if (!ok) return DQ8_OK;
    uint32_t shift = 31;  // a single block: every unit belongs to block 0
    if (p.nb > 1) {
        shift = 0;
        while (((size_t)1 << shift) < upb_l) ++shift;
    }
    const uint32_t n_full = (uint32_t)(n / U), tail = (uint32_t)(n % U);
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    if (K >= 9 && K <= 12 && !local && g_tune.avg_wide) {
        // 9 to 12 workers unrolled as well, one code word per lane and worker: units of 256 elements (K = 9: 141
        // against 156 us for the chunk kernel, K = 12: 178 against 185 us; from 13 workers on the chunk kernel wins)
        const size_t U1 = 4 * kWave, upb1 = p.B / U1;
        bool wide = p.nb == 1 || (p.B % U1 == 0 && (upb1 & (upb1 - 1)) == 0);
        wide = wide && n / U1 >= 1 && n / U1 < 0x7FFFFFFFull && ((uintptr_t)out & 15) == 0;
        for (int k = 0; k < K; ++k) wide = wide && ((uintptr_t)wp.codes[k] & 3) == 0;
        if (wide) {
            uint32_t shift1 = 31;
            if (p.nb > 1) {
                shift1 = 0;
                while (((size_t)1 << shift1) < upb1) ++shift1;
            }
            const uint32_t n_full1 = (uint32_t)(n / U1), tail1 = (uint32_t)(n % U1);
            size_t waves = (size_t)st.cus * (size_t)g_tune.avg_wide;
            if (waves > n_full1) waves = n_full1;
            const unsigned grid = (unsigned)((waves + 3) / 4);
            const uint32_t n_waves = grid * 4u;
#define DQ8_AVGW(KT)                                                                                                    \
    hipLaunchKernelGGL((k_decode_avg_full<KT, 1, 2, 4, false>), dim3(grid), dim3(kWave * 4), 0, stream, tab, wp, local, \
                       n_full1, n_waves, shift1, tail1, out)
            switch (K) {
            case 9: DQ8_AVGW(9); break;
            case 10: DQ8_AVGW(10); break;
            case 11: DQ8_AVGW(11); break;
            default: DQ8_AVGW(12); break;
            }
#undef DQ8_AVGW
            *launched = true;
            return after_launch("k_decode_avg_full", stream);
        }
    }
    if (K < 1 || K > 8 || g_tune.avg_chunk_all) {
        if (lq != 2) return DQ8_OK;  // that kernel exists for two code words per lane and worker only
        const int ch = chunk_size(K);
        // eight wavefronts per compute unit measured best for every CH from 3 up
        const int wpc = ch <= 2 ? 2 * g_tune.avg_chunk_wpc : g_tune.avg_chunk_wpc;
        size_t waves = (size_t)st.cus * (size_t)wpc;
        if (waves > n_full) waves = n_full;
        const int cw = wpc >= 8 ? 8 : 4;  // wavefronts per workgroup (they share the decode table)
        const unsigned grid = (unsigned)((waves + cw - 1) / cw);
        const uint32_t n_waves = grid * (uint32_t)cw;
        const uint64_t step = (uint64_t)n_waves * (U / 4);
        FlatGeom geom = {1, 0, 0, 0};
        if (flat_chunks) geom = FlatGeom{(uint32_t)bq, (uint32_t)(p.nb - 1), (uint32_t)(step / bq), (uint32_t)(step % bq)};
#define DQ8_CHUNK_F(CH, WPW, FL)                                                                                          \
    hipLaunchKernelGGL((k_decode_avg_chunks<CH, 2, 2, WPW, FL>), dim3(grid), dim3(kWave * WPW), 0, stream, tab, wp, K, local, \
                       n_full, n_waves, shift, geom, tail, out)
#define DQ8_CHUNK(CH, WPW) DQ8_CHUNK_F(CH, WPW, false)
        if (flat_chunks) {  // 3 to 8 workers per chunk, eight wavefronts per workgroup
            if (cw != 8) return DQ8_OK;
            switch (ch) {
            case 3: DQ8_CHUNK_F(3, 8, true); break;
            case 4: DQ8_CHUNK_F(4, 8, true); break;
            case 5: DQ8_CHUNK_F(5, 8, true); break;
            case 6: DQ8_CHUNK_F(6, 8, true); break;
            case 7: DQ8_CHUNK_F(7, 8, true); break;
            default: DQ8_CHUNK_F(8, 8, true); break;
            }
            *launched = true;
            return after_launch("k_decode_avg_chunks", stream);
        }
#define DQ8_CHUNK_W(CH)       \
    if (cw == 8) {            \
        DQ8_CHUNK(CH, 8);     \
    } else {                  \
        DQ8_CHUNK(CH, 4);     \
    }
        switch (ch) {
        case 1: DQ8_CHUNK_W(1) break;
        case 2: DQ8_CHUNK_W(2) break;
        case 3: DQ8_CHUNK_W(3) break;
        case 4: DQ8_CHUNK_W(4) break;
        case 5: DQ8_CHUNK_W(5) break;
        case 6: DQ8_CHUNK_W(6) break;
        case 7: DQ8_CHUNK_W(7) break;
        default: DQ8_CHUNK_W(8) break;
        }
#undef DQ8_CHUNK_W
#undef DQ8_CHUNK
#undef DQ8_CHUNK_F
        *launched = true;
        return after_launch("k_decode_avg_chunks", stream);
    }
    // Wavefronts per compute unit: four with 8 workers' code words in flight per lane; more with fewer workers
    // (measured per K; avg_lean_wpc scales all of them).
    static const int kWavesForK[9] = {0, 16, 8, 8, 8, 8, 4, 4, 4};
    if (flat) {
        const int fw = K <= 5 ? 8 : 4;  // wavefronts per workgroup
        // the selects between two scales make 6 and 7 workers want eight wavefronts as well (K = 7: 132 -> 121 us)
        static const int kFlatWavesForK[9] = {0, 16, 8, 8, 8, 8, 8, 8, 4};
        size_t waves = (size_t)st.cus * (size_t)(kFlatWavesForK[K] * g_tune.avg_lean_wpc / 4);
        if (waves > n_full) waves = n_full;
        const unsigned grid = (unsigned)((waves + fw - 1) / fw);
        const uint32_t n_waves = grid * (uint32_t)fw;
        const uint64_t step = (uint64_t)n_waves * (U / 4);
        const FlatGeom geom = {(uint32_t)bq, (uint32_t)(p.nb - 1), (uint32_t)(step / bq), (uint32_t)(step % bq)};
#define DQ8_AVGF(KT, WPW, LOC)                                                                                          \
    hipLaunchKernelGGL((k_decode_avg_flat<KT, 2, WPW, LOC>), dim3(grid), dim3(kWave * WPW), 0, stream, tab, wp, local, \
                       n_full, n_waves, geom, tail, out)
#define DQ8_AVGF_L(KT, WPW)        \
    if (local) {                   \
        DQ8_AVGF(KT, WPW, true);   \
    } else {                       \
        DQ8_AVGF(KT, WPW, false);  \
    }
        switch (K) {
        case 1: DQ8_AVGF_L(1, 8) break;
        case 2: DQ8_AVGF_L(2, 8) break;
        case 3: DQ8_AVGF_L(3, 8) break;
        case 4: DQ8_AVGF_L(4, 8) break;
        case 5: DQ8_AVGF_L(5, 8) break;
        case 6: DQ8_AVGF_L(6, 4) break;
        case 7: DQ8_AVGF_L(7, 4) break;
        default: DQ8_AVGF_L(8, 4) break;
        }
#undef DQ8_AVGF_L
#undef DQ8_AVGF
        *launched = true;
        return after_launch("k_decode_avg_flat", stream);
    }
    size_t waves = (size_t)st.cus * (size_t)(kWavesForK[K] * g_tune.avg_lean_wpc / 4);
    if (waves > n_full) waves = n_full;
    const unsigned grid = (unsigned)((waves + lw - 1) / lw);
    const uint32_t n_waves = grid * (uint32_t)lw;
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
    if (lq != 2 && K != 2 && K != 4 && K != 8) return DQ8_OK;  // four code words per lane: K = 2, 4, 8 only
    switch (K) {
    case 1: DQ8_AVGL_W(1, 2) break;
    case 2: DQ8_AVGL_Q(2) break;
    case 3: DQ8_AVGL_W(3, 2) break;
    case 4: DQ8_AVGL_Q(4) break;
    case 5: DQ8_AVGL_W(5, 2) break;
    case 6: DQ8_AVGL_W(6, 2) break;
    case 7: DQ8_AVGL_W(7, 2) break;
    default: DQ8_AVGL_Q(8) break;
    }
#undef DQ8_AVGL_Q
#undef DQ8_AVGL_W
#undef DQ8_AVGL_L
#undef DQ8_AVGL
    *launched = true;
    return after_launch("k_decode_avg_full", stream);
}

// K-way decode-and-average into an fp32 array with the general kernels.
int launch_decode_avg(const DeviceState &st, int kind, const WorkerPtrs &wp, int K, size_t n, size_t block, float *out,
                      hipStream_t stream)
{
    const int wpw = g_tune.avg_wpw == 16 ? 16 : (g_tune.avg_wpw == 8 ? 8 : 4);
    const bool fixed_k = K == 2 || K == 4 || K == 8;
    const size_t Bq = block_length(n, block);
    int q = K > 8 ? 1 : ((fixed_k && (g_tune.avg_q == 1 || g_tune.avg_q == 4)) ? g_tune.avg_q : 2);
    int wpc = g_tune.avg_wpc;
    fit_unit_to_block(Bq, &q, &wpc);
    Plan p = make_plan(n, block, st.cus, wpc, 1, wpw, (size_t)q * 4 * kWave);
    const uint32_t *tab = st.tables + (size_t)kind * kTableWords;
    if (g_tune.avg_lean) {
        bool launched = false;
        int rc = launch_avg_full(st, kind, wp, K, nullptr, n, p, out, stream, &launched);
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
    // The other worker counts up to 8 are unrolled too, for the default shape only; beyond that K is a loop.
#define DQ8_AVG_ODD(KT)          \
    if (q == 2 && wpw == 16) {   \
        DQ8_AVG(KT, 2, 16);      \
    } else {                     \
        DQ8_AVG_W(0, 1)          \
    }
    switch (K) {
    case 1: DQ8_AVG_ODD(1) break;
    case 2: DQ8_AVG_Q(2) break;
    case 3: DQ8_AVG_ODD(3) break;
    case 4: DQ8_AVG_Q(4) break;
    case 5: DQ8_AVG_ODD(5) break;
    case 6: DQ8_AVG_ODD(6) break;
    case 7: DQ8_AVG_ODD(7) break;
    case 8: DQ8_AVG_Q(8) break;
    default: DQ8_AVG_W(0, 1) break;
    }
#undef DQ8_AVG_ODD
#undef DQ8_AVG_Q
#undef DQ8_AVG_W
#undef DQ8_AVG
    return after_launch("k_decode_avg", stream);
}

}  // namespace

int dq8::after_launch_of(const char *what, hipStream_t stream) { return after_launch(what, stream); }

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

// ---- segments: tensors back to back in one array, one scale each

namespace {

static int check_segments(const char *who, size_t n, const uint64_t *bounds, size_t n_seg)
{
    if (!bounds) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    if (n_seg < 1 || n_seg > (size_t)kSegMax) return fail(DQ8_ERR_ARG, "%s: %zu segments outside 1..%d", who, n_seg, kSegMax);
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "%s: n too large", who);
    return DQ8_OK;
}

static int launch_segment_absmax(const DeviceState &st, const float *x, size_t n, const uint64_t *bounds, size_t n_seg,
                          float *scales, hipStream_t stream)
{
    hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((n_seg + 255) / 256)), dim3(256), 0, stream, scales, n_seg);
    int rc = after_launch("k_fill_zero", stream);
    if (rc) return rc;
    const SegPlan p = make_segment_plan(st.cus, n, n_seg, 32, true);
    const uint32_t aligned = ((uintptr_t)x & 15) == 0;
    hipLaunchKernelGGL(k_seg_absmax, dim3(p.grid), dim3(kWave * kSegWaves), p.lds, stream, x, n, bounds, (uint32_t)n_seg,
                       p.n_units, p.n_items, p.n_waves, p.group, aligned, scales);
    return after_launch("k_seg_absmax", stream);
}

}  // namespace

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
    const size_t Bq = block_length(n, block);
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(x, n * 4, codes, n) || overlaps(x, n * 4, scales, nbq * 4) || overlaps(codes, n, scales, nbq * 4))
        return fail(DQ8_ERR_ARG, "dq8_encode: buffers overlap");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool given = (flags & DQ8_SCALES_GIVEN) != 0;
    size_t done = 0;
    rc = small_encode(*st, kind, x, n, Bq, scales, codes, given, stream, &done);
    if (rc || done == n) return rc;
    x += done;  // the rest starts on a block boundary
    codes += done;
    scales += done / Bq;
    n -= done;
    // the block fits one unit: absmax and encode in one kernel
    const bool fused = !given && Bq <= (g_tune.enc_long ? kLongestHeldBlock : (size_t)kUnit);
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
    const size_t Bq = block_length(n, block);
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(out, n * 4, codes, n) || overlaps(out, n * 4, scales, nbq * 4))
        return fail(DQ8_ERR_ARG, "dq8_decode: out overlaps an input");
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    size_t done = 0;
    rc = small_decode(*st, kind, codes, scales, n, Bq, out, stream, &done);
    if (rc || done == n) return rc;
    return launch_decode(*st, kind, codes + done, scales + done / Bq, n - done, block, out + done, stream);
}

int dq8_decode_accumulate_avg(int kind, const uint8_t *const *codes, const float *const *scales, int K, size_t n,
                              size_t block, float *out, void *hip_stream)
{
    static const char who[] = "dq8_decode_accumulate_avg";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (K < 1 || K > DQ8_MAX_K) return fail(DQ8_ERR_ARG, "%s: K = %d outside 1..%d", who, K, DQ8_MAX_K);
    if (n == 0) return DQ8_OK;
    if (!codes || !scales || !out) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    if (n > (SIZE_MAX >> 3)) return fail(DQ8_ERR_ARG, "%s: n too large", who);
    const size_t Bq = block_length(n, block);
    const size_t nbq = (n + Bq - 1) / Bq;
    WorkerPtrs wp;
    rc = gather_workers(who, codes, scales, K, n, nbq, out, n * 4, &wp);
    if (rc) return rc;
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    size_t done = 0;
    rc = small_avg(*st, kind, wp, K, nullptr, n, Bq, out, stream, &done);
    if (rc || done == n) return rc;
    return launch_decode_avg(*st, kind, advance_workers(wp, K, done, Bq), K, n - done, block, out + done, stream);
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
    const size_t Bq = block_length(n, block);
    const size_t nbq = (n + Bq - 1) / Bq;
    if (overlaps(out, n * 4, local, n * 4)) return fail(DQ8_ERR_ARG, "%s: out overlaps local", who);
    WorkerPtrs wp;
    rc = gather_workers(who, codes, scales, K, n, nbq, out, n * 4, &wp);
    if (rc) return rc;
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    size_t done = 0;
    rc = small_avg(*st, kind, wp, K, local, n, Bq, out, stream, &done);
    if (rc || done == n) return rc;
    if (done) {  // the rest starts on a block boundary
        wp = advance_workers(wp, K, done, Bq);
        local += done;
        out += done;
        n -= done;
    }
    if (g_tune.avg_lean) {
        const Plan p = make_plan(n, block, st->cus, 1, 1);
        bool launched = false;
        rc = launch_avg_full(*st, kind, wp, K, local, n, p, out, stream, &launched);
        if (rc || launched) return rc;
    }
    return launch_avg_block(*st, kind, wp, K, local, n, block, out, nullptr, nullptr, stream);
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
    const size_t Bq = block_length(n, block);
    const size_t nbq = (n + Bq - 1) / Bq;
    if (Bq > kLongestHeldBlock)
        return fail(DQ8_ERR_ARG, "%s: a scale block of %zu elements does not fit the registers of a workgroup (at most %zu); "
                    "use dq8_decode_accumulate_avg and dq8_encode", who, Bq, kLongestHeldBlock);
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
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (Bq > (size_t)kUnit) return launch_avg_long(*st, kind, wp, K, local, n, block, out_scales, out_codes, stream);
    size_t done = 0;
    // (blocks of 1024 elements: a wavefront per block is faster where that kernel exists for the worker count)
    if (!(Bq == 1024 && short_team_k(K, Bq) && g_tune.avg_team)) rc = small_avg_encode(*st, kind, wp, K, local, n, Bq, out_scales, out_codes, stream, &done);
    if (rc || done == n) return rc;
    if (done) {  // the rest starts on a block boundary
        wp = advance_workers(wp, K, done, Bq);
        if (local) local += done;
        out_codes += done;
        out_scales += done / Bq;
        n -= done;
    }
    return launch_avg_block(*st, kind, wp, K, local, n, block, nullptr, out_scales, out_codes, stream);
}

int dq8_absmax_segments(const float *x, size_t n, const uint64_t *bounds, size_t n_seg, float *scales, void *hip_stream)
{
    static const char who[] = "dq8_absmax_segments";
    if (n == 0) return DQ8_OK;
    if (!x || !scales) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    int rc = check_segments(who, n, bounds, n_seg);
    if (rc) return rc;
    if (overlaps(x, n * 4, scales, n_seg * 4) || overlaps(bounds, (n_seg + 1) * 8, scales, n_seg * 4))
        return fail(DQ8_ERR_ARG, "%s: buffers overlap", who);
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    return launch_segment_absmax(*st, x, n, bounds, n_seg, scales, static_cast<hipStream_t>(hip_stream));
}

int dq8_encode_segments(int kind, const float *x, size_t n, const uint64_t *bounds, size_t n_seg, float *scales,
                        uint8_t *codes, unsigned flags, void *hip_stream)
{
    static const char who[] = "dq8_encode_segments";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (flags & ~DQ8_SCALES_GIVEN) return fail(DQ8_ERR_ARG, "%s: unknown flags 0x%x", who, flags);
    if (n == 0) return DQ8_OK;
    if (!x || !scales || !codes) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    rc = check_segments(who, n, bounds, n_seg);
    if (rc) return rc;
    if (overlaps(x, n * 4, codes, n) || overlaps(x, n * 4, scales, n_seg * 4) || overlaps(codes, n, scales, n_seg * 4) ||
        overlaps(bounds, (n_seg + 1) * 8, codes, n) || overlaps(bounds, (n_seg + 1) * 8, scales, n_seg * 4))
        return fail(DQ8_ERR_ARG, "%s: buffers overlap", who);
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!(flags & DQ8_SCALES_GIVEN)) {
        rc = launch_segment_absmax(*st, x, n, bounds, n_seg, scales, stream);
        if (rc) return rc;
    }
    SegPlan p = make_segment_plan(st->cus, n, n_seg, 32);
    p.lds += (size_t)st->search_words[kind] * sizeof(uint32_t);
    const uint32_t aligned = (((uintptr_t)x & 15) | ((uintptr_t)codes & 3)) == 0;
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    if (st->has_remap[kind])
        hipLaunchKernelGGL((k_seg_encode<true>), dim3(p.grid), dim3(kWave * kSegWaves), p.lds, stream, tab, x, n, bounds,
                           (uint32_t)n_seg, p.n_units, p.n_waves, aligned, scales, codes);
    else
        hipLaunchKernelGGL((k_seg_encode<false>), dim3(p.grid), dim3(kWave * kSegWaves), p.lds, stream, tab, x, n, bounds,
                           (uint32_t)n_seg, p.n_units, p.n_waves, aligned, scales, codes);
    return after_launch("k_seg_encode", stream);
}

int dq8_decode_segments(int kind, const uint8_t *codes, const float *scales, size_t n, const uint64_t *bounds, size_t n_seg,
                        float *out, void *hip_stream)
{
    static const char who[] = "dq8_decode_segments";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (n == 0) return DQ8_OK;
    if (!codes || !scales || !out) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    rc = check_segments(who, n, bounds, n_seg);
    if (rc) return rc;
    if (overlaps(out, n * 4, codes, n) || overlaps(out, n * 4, scales, n_seg * 4) || overlaps(out, n * 4, bounds, (n_seg + 1) * 8))
        return fail(DQ8_ERR_ARG, "%s: out overlaps an input", who);
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const SegPlan p = make_segment_plan(st->cus, n, n_seg, 16);
    const uint32_t aligned = (((uintptr_t)out & 15) | ((uintptr_t)codes & 3)) == 0;
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    hipLaunchKernelGGL(k_seg_decode, dim3(p.grid), dim3(kWave * kSegWaves), p.lds, stream, tab, codes, scales, n, bounds,
                       (uint32_t)n_seg, p.n_units, p.n_waves, aligned, out);
    return after_launch("k_seg_decode", stream);
}

int dq8_decode_accumulate_avg_segments(int kind, const uint8_t *const *codes, const float *const *scales, int K,
                                       const float *local, size_t n, const uint64_t *bounds, size_t n_seg, float *out,
                                       void *hip_stream)
{
    static const char who[] = "dq8_decode_accumulate_avg_segments";
    int rc = check_kind(kind);
    if (rc) return rc;
    if (K < (local ? 0 : 1) || K > DQ8_MAX_K)
        return fail(DQ8_ERR_ARG, "%s: K = %d outside %d..%d", who, K, local ? 0 : 1, DQ8_MAX_K);
    if (n == 0) return DQ8_OK;
    if (!out) return fail(DQ8_ERR_NULL, "%s: NULL pointer", who);
    rc = check_segments(who, n, bounds, n_seg);
    if (rc) return rc;
    if (overlaps(out, n * 4, bounds, (n_seg + 1) * 8)) return fail(DQ8_ERR_ARG, "%s: out overlaps the offsets", who);
    if (local && overlaps(out, n * 4, local, n * 4)) return fail(DQ8_ERR_ARG, "%s: out overlaps local", who);
    WorkerPtrs wp;
    rc = gather_workers(who, codes, scales, K, n, n_seg, out, n * 4, &wp);
    if (rc) return rc;
    DeviceState *st;
    rc = device_state(&st);
    if (rc) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const SegPlan p = make_segment_plan(st->cus, n, n_seg, 16);
    bool aligned = ((uintptr_t)out & 15) == 0 && ((uintptr_t)local & 15) == 0;
    for (int k = 0; k < K; ++k) aligned = aligned && ((uintptr_t)wp.codes[k] & 3) == 0;
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    hipLaunchKernelGGL(k_seg_avg, dim3(p.grid), dim3(kWave * kSegWaves), p.lds, stream, tab, wp, K, local, n, bounds,
                       (uint32_t)n_seg, p.n_units, p.n_waves, (uint32_t)aligned, out);
    return after_launch("k_seg_avg", stream);
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
    const size_t Bq = block_length(n, block);
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

int dq8_internal_chunk_size(int K) { return chunk_size(K); }

int dq8_internal_units(size_t n, size_t block, int quads, int waves_per_cu, size_t *out4)
{
    if (!out4 || quads < 1 || quads > 16 || (quads & (quads - 1)) || waves_per_cu < 1 || n == 0)
        return fail(DQ8_ERR_ARG, "dq8_internal_units: bad argument");
    const size_t Bq = block_length(n, block);
    fit_unit_to_block(Bq, &quads, &waves_per_cu);
    out4[0] = Bq;
    out4[1] = (size_t)quads * 4 * kWave;
    out4[2] = (size_t)waves_per_cu;
    out4[3] = holding_unit(Bq);
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
#ifndef DQ8_TUNABLE
    (void)value;
    return fail(DQ8_ERR_ARG, "dq8_internal_tune: this build has fixed launch shapes (compile with -DDQ8_TUNABLE)");
#else
    struct { const char *name; int *slot; int lo, hi; } keys[] = {
        {"amax_nt", &g_tune.amax_nt, 0, 1}, 
        {"avg_lean", &g_tune.avg_lean, 0, 1}, {"avg_lean_q", &g_tune.avg_lean_q, 2, 4},
        {"avg_lean_wpc", &g_tune.avg_lean_wpc, 1, 32}, {"avg_chunk_wpc", &g_tune.avg_chunk_wpc, 1, 32}, {"avg_chunk_all", &g_tune.avg_chunk_all, 0, 1}, {"avg_wide", &g_tune.avg_wide, 0, 32}, {"avg_flat", &g_tune.avg_flat, 0, 1}, {"avg_lean_wpw", &g_tune.avg_lean_wpw, 4, 16}, {"copy_nt", &g_tune.copy_nt, 0, 2},           {"fastdiv", &g_tune.fastdiv, 0, 1},   {"enc_wpb", &g_tune.enc_wpb, 1, 4},
        {"enc_long", &g_tune.enc_long, 0, 2}, {"enc_wpc12", &g_tune.enc_wpc12, 4, 32}, {"enc_wpc6", &g_tune.enc_wpc6, 4, 32}, {"enc_wpc4", &g_tune.enc_wpc4, 4, 32}, {"enc_mid", &g_tune.enc_mid, 0, 4095}, {"enc_wave", &g_tune.enc_wave, 0, 2048}, {"enc_wave_min", &g_tune.enc_wave_min, 4, 2048}, {"enc_wave_wpc", &g_tune.enc_wave_wpc, 4, 32}, {"enc_wave_wpc8", &g_tune.enc_wave_wpc8, 4, 32}, {"enc_wpc8", &g_tune.enc_wpc8, 4, 32}, {"enc_wpc16", &g_tune.enc_wpc16, 4, 32},
        {"enc_wpc", &g_tune.enc_wpc, 1, 32}, {"enc_lean", &g_tune.enc_lean, 0, 1}, {"enc_lean_wpc", &g_tune.enc_lean_wpc, 4, 32}, {"enc_fill", &g_tune.enc_fill, 0, 1}, {"amax_q", &g_tune.amax_q, 1, 16},    {"amax_wpc", &g_tune.amax_wpc, 1, 32}, {"amax_waste", &g_tune.amax_waste, 0, 1},
        {"dec_flat", &g_tune.dec_flat, 0, 2}, {"dec_q", &g_tune.dec_q, 1, 16},     {"dec_wpc", &g_tune.dec_wpc, 1, 32},  {"avg_q", &g_tune.avg_q, 1, 4},
        {"avg_wpc", &g_tune.avg_wpc, 1, 32}, {"avg_wpw", &g_tune.avg_wpw, 4, 16}, {"dec_wpw", &g_tune.dec_wpw, 4, 16}, {"blk_wpw", &g_tune.blk_wpw, 6, 8}, {"avg_team", &g_tune.avg_team, 0, 1}, {"avg_steady", &g_tune.avg_steady, 0, 1}, {"avg_teams", &g_tune.avg_teams, 0, 4}, {"avg_teams4_upto", &g_tune.avg_teams4_upto, 0, 6}, {"avg_wgpc", &g_tune.avg_wgpc, 1, 2}, {"copy_q", &g_tune.copy_q, 1, 16},    {"copy_wpc", &g_tune.copy_wpc, 1, 32},
    };
    for (auto &k : keys)
        if (!std::strcmp(k.name, key)) {
            if (value < k.lo || value > k.hi) return fail(DQ8_ERR_ARG, "dq8_internal_tune: %s = %d outside %d..%d", key, value, k.lo, k.hi);
            *k.slot = value;
            return DQ8_OK;
        }
    return fail(DQ8_ERR_ARG, "dq8_internal_tune: unknown key %s", key);
#endif
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
    return after_launch("k_copy", stream);
}

int dq8_internal_device_info(int *out5)
{
    if (!out5) return fail(DQ8_ERR_NULL, "dq8_internal_device_info: out5 is NULL");
    int dev = -1;
    DQ8_HIP(hipGetDevice(&dev));
    const hipDeviceAttribute_t what[5] = {hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate,
                                          hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth,
                                          hipDeviceAttributeL2CacheSize};
    for (int i = 0; i < 5; ++i) DQ8_HIP(hipDeviceGetAttribute(&out5[i], what[i], dev));
    return DQ8_OK;
}

static int host_search(int kind, Search *sr)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    *sr = make_search(t.bucket, t.lo_key, t.n_bucket, t.has_marks);
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
        const uint32_t want = t.canon[j];
        // the lookup for a correctly rounded quotient is right for every value
        bad += code_of(sr, search_sum_exact(sr, pos), pos) != want;
        bad += code_of(sr, search_sum_exact(sr, neg), neg) != (want | 0x80u);
        // the lookup for a product x * fl(1 / s) is right wherever it does not raise the proximity flag,
        const uint32_t sp = search_sum(sr, pos), sn = search_sum(sr, neg);
        if (near_key(sp) > 2 * kNearWindow) bad += code_of(sr, sp, pos) != want;
        if (near_key(sn) > 2 * kNearWindow) bad += code_of(sr, sn, neg) != (want | 0x80u);
        // and every value within kNearWindow steps of a threshold raises it
        bool close = (j < n_thr && thr_bits[j] - bits <= kNearWindow) || (j > 0 && bits - thr_bits[j - 1] <= kNearWindow);
        if (close && (near_key(sp) > 2 * kNearWindow || near_key(sn) > 2 * kNearWindow)) ++missed;
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
