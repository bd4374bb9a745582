// dq8 kernels and C ABI for gfx950 (MI355X).  See include/dq8.h for the contract.
//
// Work decomposition shared by every kernel: the array is cut into UNITS.  A unit is
// a run of at most kUnit consecutive elements that lies inside one scale block, so
// one scale applies to the whole unit: unit u = (block b, chunk c) covers elements
// [b*B + c*kUnit, min(b*B + (c+1)*kUnit, (b+1)*B, n)).  One 64-lane wavefront owns a
// unit at a time and walks units with a grid-wide stride; the host sizes the grid so
// that every wavefront gets the same number of units and all of them are resident.
//
// Inside a unit lane L owns elements 4*(64*it + L) .. +3 for it = 0..15: fp32 data
// moves as one 128-bit access per lane (1 KiB contiguous per wave instruction) and
// the matching four codes as one 32-bit access (256 B contiguous per instruction).
// Units that are short, or whose addresses are not aligned for that, take a plain
// strided element loop with identical arithmetic.
//
// Built with -ffp-contract=off: the decode-and-average sum must round the product
// and the sum separately.  Divisions are the compiler's correctly rounded ones.
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
using dq8::kCbOff;
using dq8::kLoKeyOff;
using dq8::kNBucketOff;
using dq8::kTableWords;

constexpr int kWave = 64;
constexpr int kWavesPerWg = 4;
constexpr int kWg = kWave * kWavesPerWg;
constexpr int kUnit = 4096;            // elements per unit
constexpr int kQuadIters = kUnit / (4 * kWave);  // 16 quads per lane per unit
constexpr int kKinds = 3;
constexpr int kLutCopies = 32;         // one copy of the decode table per LDS bank

// Tables of the three data types, one image per device (each GPU holds its own copy).
__device__ __align__(256) uint32_t g_tables[kKinds][kTableWords];

struct WorkerPtrs {
    const uint8_t *codes[DQ8_MAX_K];
    const float *scales[DQ8_MAX_K];
};

// ---------------------------------------------------------------- device helpers

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, m, kWave);
        v = o > v ? o : v;
    }
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}

__device__ __forceinline__ uint32_t abs_bits(float f) { return __float_as_uint(f) & 0x7FFFFFFFu; }

// Geometry of unit u.  All values are wave-uniform.
struct Unit {
    size_t block;   // scale index
    size_t start;   // first element
    uint32_t len;   // 1..kUnit
};

__device__ __forceinline__ Unit unit_of(size_t u, size_t n, size_t B, size_t upb)
{
    Unit r;
    size_t c;
    if (upb == 1) {
        r.block = u;
        c = 0;
    } else if (B >= n) {
        r.block = 0;
        c = u;
    } else {
        r.block = u / upb;
        c = u - r.block * upb;
    }
    size_t off = c * (size_t)kUnit;
    r.start = r.block * B + off;
    size_t len = B - off;
    if (len > (size_t)kUnit) len = kUnit;
    if (len > n - r.start) len = n - r.start;
    r.len = (uint32_t)len;
    return r;
}

// Search state for the encoder: bucket table in LDS plus its key range.
struct Search {
    const uint32_t *bucket;  // LDS
    uint32_t lo_key, hi_key;
};

// Code of the normalised value xn: magnitude index = number of thresholds <= |xn|
// (nearest table magnitude, ties to the smaller), bit 7 = sign bit of xn.
__host__ __device__ __forceinline__ uint32_t code_of(const Search &s, float xn)
{
    uint32_t bits;
    __builtin_memcpy(&bits, &xn, 4);
    uint32_t key = (bits >> 16) & 0x7FFFu;
    key = key < s.lo_key ? s.lo_key : key;
    key = key > s.hi_key ? s.hi_key : key;
    uint32_t e = s.bucket[key - s.lo_key];
    uint32_t mag = (e + (bits & 0xFFFFu)) >> 16;
    return mag | ((bits >> 24) & 0x80u);
}

__device__ __forceinline__ void load_bucket_table(const uint32_t *tab, uint32_t *lds, Search *s)
{
    uint32_t nbk = tab[kNBucketOff];
    for (uint32_t i = threadIdx.x; i < nbk; i += kWg) lds[i] = tab[kBucketOff + i];
    s->bucket = lds;
    s->lo_key = tab[kLoKeyOff];
    s->hi_key = s->lo_key + nbk - 1;
    __syncthreads();
}

// Decode table replicated once per LDS bank: entry (code, copy) at code * 32 + copy.
__device__ __forceinline__ void load_lut(const uint32_t *tab, float *lds)
{
    for (uint32_t i = threadIdx.x; i < 256 * kLutCopies; i += kWg)
        lds[i] = __uint_as_float(tab[kCbOff + (i / kLutCopies)]);
    __syncthreads();
}

// Index of this wavefront in the grid = the first unit it owns; held in scalar registers.
__device__ __forceinline__ size_t first_unit()
{
    uint32_t w = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    return (size_t)blockIdx.x * kWavesPerWg + w;
}

// ---------------------------------------------------------------- kernels

__global__ void k_fill_zero(float *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

// Plain fp32 copy with the access pattern of the codec kernels (one unit per wavefront step,
// 128-bit accesses).  Exists to calibrate bandwidth and hardware-counter readings against a
// kernel whose traffic is known exactly: 4 bytes read and 4 bytes written per element.
__global__ __launch_bounds__(kWg) void k_copy(const float *__restrict__ src, float *__restrict__ dst, size_t n,
                                             size_t n_units, size_t n_waves)
{
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of(u, n, n, 0);
        const float *ps = src + un.start;
        float *pd = dst + un.start;
        if (un.len == kUnit && (((uintptr_t)ps | (uintptr_t)pd) & 15) == 0) {
            const float4 *s4 = reinterpret_cast<const float4 *>(ps);
            float4 *d4 = reinterpret_cast<float4 *>(pd);
            float4 v[kQuadIters];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) v[it] = s4[it * kWave + lane];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) d4[it * kWave + lane] = v[it];
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) pd[i] = ps[i];
        }
    }
}

// Block maxima.  upb == 1: each unit is a whole block and stores its maximum.
// upb > 1: scales[] was zeroed and the units of a block merge with an integer atomic max
// (non-negative binary32 numbers order like their bit patterns).
__global__ __launch_bounds__(kWg) void k_absmax(const float *__restrict__ x, size_t n, size_t B, size_t upb,
                                               size_t n_units, size_t n_waves, float *__restrict__ scales)
{
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of(u, n, B, upb);
        const float *px = x + un.start;
        uint32_t m = 0;
        if (un.len == kUnit && ((uintptr_t)px & 15) == 0) {
            const float4 *p4 = reinterpret_cast<const float4 *>(px);
            float4 v[kQuadIters];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) v[it] = p4[it * kWave + lane];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) {
                uint32_t a = abs_bits(v[it].x), b = abs_bits(v[it].y), c = abs_bits(v[it].z), d = abs_bits(v[it].w);
                a = a > b ? a : b;
                c = c > d ? c : d;
                a = a > c ? a : c;
                m = m > a ? m : a;
            }
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) {
                uint32_t a = abs_bits(px[i]);
                m = m > a ? m : a;
            }
        }
        m = wave_max_u32(m);
        if (lane == 0) {
            if (upb == 1)
                scales[un.block] = __uint_as_float(m);
            else
                atomicMax(reinterpret_cast<unsigned int *>(scales) + un.block, m);
        }
    }
}

// Compression.  FUSED: a unit is a whole block (upb == 1); the wave reduces the block's
// maximum from registers, stores it and quantises the same registers.  Otherwise the
// scale of the unit's block is read from scales[].
template <bool FUSED>
__global__ __launch_bounds__(kWg) void k_encode(const uint32_t *__restrict__ tab, const float *__restrict__ x, size_t n,
                                               size_t B, size_t upb, size_t n_units, size_t n_waves,
                                               float *__restrict__ scales, uint8_t *__restrict__ codes)
{
    extern __shared__ uint32_t lds_bucket[];
    Search sr;
    load_bucket_table(tab, lds_bucket, &sr);
    const uint32_t lane = threadIdx.x & 63;
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of(u, n, B, upb);
        const float *px = x + un.start;
        uint8_t *pc = codes + un.start;
        if (un.len == kUnit && ((uintptr_t)px & 15) == 0 && ((uintptr_t)pc & 3) == 0) {
            const float4 *p4 = reinterpret_cast<const float4 *>(px);
            uint32_t *c4 = reinterpret_cast<uint32_t *>(pc);
            float4 v[kQuadIters];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) v[it] = p4[it * kWave + lane];
            float s;
            if (FUSED) {
                uint32_t m = 0;
#pragma unroll
                for (int it = 0; it < kQuadIters; ++it) {
                    uint32_t a = abs_bits(v[it].x), b = abs_bits(v[it].y), c = abs_bits(v[it].z), d = abs_bits(v[it].w);
                    a = a > b ? a : b;
                    c = c > d ? c : d;
                    a = a > c ? a : c;
                    m = m > a ? m : a;
                }
                s = __uint_as_float(wave_max_u32(m));
                if (lane == 0) scales[un.block] = s;
            } else {
                s = scales[un.block];
            }
            const float d = s == 0.0f ? 1.0f : s;  // a zero scale leaves the value as it is
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) {
                uint32_t w = code_of(sr, v[it].x / d) | (code_of(sr, v[it].y / d) << 8) |
                             (code_of(sr, v[it].z / d) << 16) | (code_of(sr, v[it].w / d) << 24);
                c4[it * kWave + lane] = w;
            }
        } else {
            float s;
            if (FUSED) {
                uint32_t m = 0;
                for (uint32_t i = lane; i < un.len; i += kWave) {
                    uint32_t a = abs_bits(px[i]);
                    m = m > a ? m : a;
                }
                s = __uint_as_float(wave_max_u32(m));
                if (lane == 0) scales[un.block] = s;
            } else {
                s = scales[un.block];
            }
            const float d = s == 0.0f ? 1.0f : s;
            for (uint32_t i = lane; i < un.len; i += kWave) pc[i] = (uint8_t)code_of(sr, px[i] / d);
        }
    }
}

// Decompression of one buffer: out = table[code] * scale.
__global__ __launch_bounds__(kWg) void k_decode(const uint32_t *__restrict__ tab, const uint8_t *__restrict__ codes,
                                               const float *__restrict__ scales, size_t n, size_t B, size_t upb,
                                               size_t n_units, size_t n_waves, float *__restrict__ out)
{
    __shared__ float lut[256 * kLutCopies];
    load_lut(tab, lut);
    const uint32_t lane = threadIdx.x & 63;
    const float *my = lut + (lane & (kLutCopies - 1));
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of(u, n, B, upb);
        const uint8_t *pc = codes + un.start;
        float *po = out + un.start;
        const float s = scales[un.block];
        if (un.len == kUnit && ((uintptr_t)po & 15) == 0 && ((uintptr_t)pc & 3) == 0) {
            const uint32_t *c4 = reinterpret_cast<const uint32_t *>(pc);
            float4 *o4 = reinterpret_cast<float4 *>(po);
            uint32_t w[kQuadIters];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) w[it] = c4[it * kWave + lane];
#pragma unroll
            for (int it = 0; it < kQuadIters; ++it) {
                float4 r;
                r.x = my[(w[it] & 0xFFu) * kLutCopies] * s;
                r.y = my[((w[it] >> 8) & 0xFFu) * kLutCopies] * s;
                r.z = my[((w[it] >> 16) & 0xFFu) * kLutCopies] * s;
                r.w = my[(w[it] >> 24) * kLutCopies] * s;
                o4[it * kWave + lane] = r;
            }
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) po[i] = my[(uint32_t)pc[i] * kLutCopies] * s;
        }
    }
}

// Decompress K buffers and average: acc = +0; acc += table[code_k] * scale_k for k = 0..K-1
// in order; out = acc / K.  KT > 0 fixes K at compile time (fully unrolled), KT == 0 reads it.
template <int KT>
__global__ __launch_bounds__(kWg) void k_decode_avg(const uint32_t *__restrict__ tab, WorkerPtrs p, int K_rt, size_t n,
                                                   size_t B, size_t upb, size_t n_units, size_t n_waves,
                                                   float *__restrict__ out)
{
    __shared__ float lut[256 * kLutCopies];
    load_lut(tab, lut);
    const int K = KT > 0 ? KT : K_rt;
    const float fk = (float)K;
    const uint32_t lane = threadIdx.x & 63;
    const float *my = lut + (lane & (kLutCopies - 1));
    constexpr int kSub = 4;  // quads per lane kept in flight per worker
    for (size_t u = first_unit(); u < n_units; u += n_waves) {
        Unit un = unit_of(u, n, B, upb);
        float *po = out + un.start;
        bool fast = un.len == kUnit && ((uintptr_t)po & 15) == 0;
        if (KT > 0) {
#pragma unroll
            for (int k = 0; k < KT; ++k) fast = fast && (((uintptr_t)(p.codes[k] + un.start) & 3) == 0);
        } else {
            for (int k = 0; k < K; ++k) fast = fast && (((uintptr_t)(p.codes[k] + un.start) & 3) == 0);
        }
        if (fast) {
            float4 *o4 = reinterpret_cast<float4 *>(po);
            if (KT > 0) {
                float sc[KT > 0 ? KT : 1];
#pragma unroll
                for (int k = 0; k < KT; ++k) sc[k] = p.scales[k][un.block];
                for (int sub = 0; sub < kQuadIters / kSub; ++sub) {
                    uint32_t w[KT > 0 ? KT : 1][kSub];
#pragma unroll
                    for (int k = 0; k < KT; ++k) {
                        const uint32_t *c4 = reinterpret_cast<const uint32_t *>(p.codes[k] + un.start);
#pragma unroll
                        for (int j = 0; j < kSub; ++j) w[k][j] = c4[(sub * kSub + j) * kWave + lane];
                    }
#pragma unroll
                    for (int j = 0; j < kSub; ++j) {
                        float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
                        for (int k = 0; k < KT; ++k) {
                            a.x = a.x + my[(w[k][j] & 0xFFu) * kLutCopies] * sc[k];
                            a.y = a.y + my[((w[k][j] >> 8) & 0xFFu) * kLutCopies] * sc[k];
                            a.z = a.z + my[((w[k][j] >> 16) & 0xFFu) * kLutCopies] * sc[k];
                            a.w = a.w + my[(w[k][j] >> 24) * kLutCopies] * sc[k];
                        }
                        a.x = a.x / fk;
                        a.y = a.y / fk;
                        a.z = a.z / fk;
                        a.w = a.w / fk;
                        o4[(sub * kSub + j) * kWave + lane] = a;
                    }
                }
            } else {
                for (int it = 0; it < kQuadIters; ++it) {
                    float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    for (int k = 0; k < K; ++k) {
                        const uint32_t w = reinterpret_cast<const uint32_t *>(p.codes[k] + un.start)[it * kWave + lane];
                        const float s = p.scales[k][un.block];
                        a.x = a.x + my[(w & 0xFFu) * kLutCopies] * s;
                        a.y = a.y + my[((w >> 8) & 0xFFu) * kLutCopies] * s;
                        a.z = a.z + my[((w >> 16) & 0xFFu) * kLutCopies] * s;
                        a.w = a.w + my[(w >> 24) * kLutCopies] * s;
                    }
                    a.x = a.x / fk;
                    a.y = a.y / fk;
                    a.z = a.z / fk;
                    a.w = a.w / fk;
                    o4[it * kWave + lane] = a;
                }
            }
        } else {
            for (uint32_t i = lane; i < un.len; i += kWave) {
                float a = 0.0f;
                for (int k = 0; k < K; ++k) a = a + my[(uint32_t)p.codes[k][un.start + i] * kLutCopies] * p.scales[k][un.block];
                po[i] = a / fk;
            }
        }
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
    uint32_t n_bucket[kKinds] = {0, 0, 0};
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
            st.n_bucket[k] = t.n_bucket;
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

int tune_waves_per_cu()
{
    static int v = [] {
        const char *e = getenv("DQ8_WAVES_PER_CU");
        int w = e ? atoi(e) : 0;
        return (w >= 1 && w <= 32) ? w : 16;
    }();
    return v;
}

struct Plan {
    size_t B, nb, upb, n_units, n_waves;
    unsigned grid;
};

// Units, and a grid in which every wavefront walks the same number of them.
Plan make_plan(size_t n, size_t block, const DeviceState &st)
{
    Plan p;
    p.B = (block == 0 || block > n) ? n : block;
    p.nb = (n + p.B - 1) / p.B;
    p.upb = (p.B + kUnit - 1) / kUnit;
    if (p.nb == 1) {
        p.n_units = (n + kUnit - 1) / kUnit;
    } else {
        size_t last = n - (p.nb - 1) * p.B;  // the last block may be short
        p.n_units = (p.nb - 1) * p.upb + (last + kUnit - 1) / kUnit;
    }
    size_t max_waves = (size_t)st.cus * (size_t)tune_waves_per_cu();
    size_t per_wave = (p.n_units + max_waves - 1) / max_waves;
    size_t waves = (p.n_units + per_wave - 1) / per_wave;
    size_t grid = (waves + kWavesPerWg - 1) / kWavesPerWg;
    p.grid = (unsigned)grid;
    p.n_waves = grid * kWavesPerWg;
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
    Plan p = make_plan(n, block, st);
    if (p.upb > 1) {
        unsigned g = (unsigned)((p.nb + 255) / 256);
        hipLaunchKernelGGL(k_fill_zero, dim3(g), dim3(256), 0, stream, scales, p.nb);
        int rc = after_launch("k_fill_zero");
        if (rc) return rc;
    }
    hipLaunchKernelGGL(k_absmax, dim3(p.grid), dim3(kWg), 0, stream, x, n, p.B, p.upb, p.n_units, p.n_waves, scales);
    return after_launch("k_absmax");
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
    Plan p = make_plan(n, block, *st);
    if (overlaps(x, n * 4, codes, n) || overlaps(x, n * 4, scales, p.nb * 4) || overlaps(codes, n, scales, p.nb * 4))
        return fail(DQ8_ERR_ARG, "dq8_encode: buffers overlap");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    const size_t lds = (size_t)st->n_bucket[kind] * sizeof(uint32_t);
    const bool given = (flags & DQ8_SCALES_GIVEN) != 0;
    if (!given && p.upb == 1) {
        hipLaunchKernelGGL(k_encode<true>, dim3(p.grid), dim3(kWg), lds, stream, tab, x, n, p.B, p.upb, p.n_units,
                           p.n_waves, scales, codes);
        return after_launch("k_encode<fused>");
    }
    if (!given) {
        rc = launch_absmax(*st, x, n, block, scales, stream);
        if (rc) return rc;
    }
    hipLaunchKernelGGL(k_encode<false>, dim3(p.grid), dim3(kWg), lds, stream, tab, x, n, p.B, p.upb, p.n_units,
                       p.n_waves, scales, codes);
    return after_launch("k_encode<scales>");
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
    Plan p = make_plan(n, block, *st);
    if (overlaps(out, n * 4, codes, n) || overlaps(out, n * 4, scales, p.nb * 4))
        return fail(DQ8_ERR_ARG, "dq8_decode: out overlaps an input");
    const uint32_t *tab = st->tables + (size_t)kind * kTableWords;
    hipLaunchKernelGGL(k_decode, dim3(p.grid), dim3(kWg), 0, static_cast<hipStream_t>(hip_stream), tab, codes, scales, n,
                       p.B, p.upb, p.n_units, p.n_waves, out);
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
    Plan p = make_plan(n, block, *st);
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
#define DQ8_LAUNCH_AVG(KT)                                                                                             \
    hipLaunchKernelGGL(k_decode_avg<KT>, dim3(p.grid), dim3(kWg), 0, stream, tab, wp, K, n, p.B, p.upb, p.n_units,   \
                       p.n_waves, out)
    switch (K) {
    case 2: DQ8_LAUNCH_AVG(2); break;
    case 4: DQ8_LAUNCH_AVG(4); break;
    case 8: DQ8_LAUNCH_AVG(8); break;
    default: DQ8_LAUNCH_AVG(0); break;
    }
#undef DQ8_LAUNCH_AVG
    return after_launch("k_decode_avg");
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

int dq8_internal_plan(size_t n, size_t block, int cus, size_t *out6)
{
    DeviceState st;
    st.cus = cus;
    Plan p = make_plan(n, block, st);
    out6[0] = p.B;
    out6[1] = p.nb;
    out6[2] = p.upb;
    out6[3] = p.n_units;
    out6[4] = p.n_waves;
    out6[5] = p.grid;
    return DQ8_OK;
}

int dq8_internal_copy(float *dst, const float *src, size_t n, void *hip_stream)
{
    if (n == 0) return DQ8_OK;
    if (!dst || !src) return fail(DQ8_ERR_NULL, "dq8_internal_copy: NULL pointer");
    DeviceState *st;
    int rc = device_state(&st);
    if (rc) return rc;
    Plan p = make_plan(n, 0, *st);
    hipLaunchKernelGGL(k_copy, dim3(p.grid), dim3(kWg), 0, static_cast<hipStream_t>(hip_stream), src, dst, n, p.n_units,
                       p.n_waves);
    return after_launch("k_copy");
}

static int host_search(int kind, Search *sr, const dq8::Tables **tp)
{
    int rc = check_kind(kind);
    if (rc) return rc;
    static thread_local dq8::Tables t;
    if (dq8::build_tables(kind, &t)) return fail(DQ8_ERR_KIND, "table construction failed for kind %d", kind);
    sr->bucket = t.bucket;
    sr->lo_key = t.lo_key;
    sr->hi_key = t.lo_key + t.n_bucket - 1;
    *tp = &t;
    return DQ8_OK;
}

int dq8_internal_check_search(int kind, uint64_t *mismatches)
{
    Search sr;
    const dq8::Tables *t;
    int rc = host_search(kind, &sr, &t);
    if (rc) return rc;
    uint32_t thr_bits[127];
    std::memcpy(thr_bits, t->thr, sizeof(thr_bits));
    uint64_t bad = 0;
    uint32_t j = 0;  // thresholds <= the current value
    for (uint32_t bits = 0; bits <= 0x7F800000u; ++bits) {
        while (j < 127 && thr_bits[j] <= bits) ++j;
        float pos, neg;
        uint32_t nb = bits | 0x80000000u;
        std::memcpy(&pos, &bits, 4);
        std::memcpy(&neg, &nb, 4);
        bad += code_of(sr, pos) != j;
        bad += code_of(sr, neg) != (j | 0x80u);
    }
    *mismatches = bad;
    return DQ8_OK;
}

int dq8_internal_search(int kind, const float *xn, size_t n, uint8_t *codes)
{
    Search sr;
    const dq8::Tables *t;
    int rc = host_search(kind, &sr, &t);
    if (rc) return rc;
    for (size_t i = 0; i < n; ++i) codes[i] = (uint8_t)code_of(sr, xn[i]);
    return DQ8_OK;
}

}  // extern "C"
