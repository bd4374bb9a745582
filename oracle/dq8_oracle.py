"""numpy front end of the C oracle (dq8_oracle.c) -- test infrastructure, not the product.

Argument marshalling only: every number comes out of the C file, which is built
with ``gcc -O2 -fno-fast-math -ffp-contract=off`` so that each fp32 operation is
rounded once and never fused.  The functions follow Sec. 3.1 (data types, absmax
normalisation), Sec. 3.2 (compression / decompression) and Sec. 2.1 (averaging)
of arXiv 1511.04561.
"""
import ctypes
import os
import subprocess

import numpy as np

DYNAMIC_TREE, LINEAR, STATIC_TREE, MANTISSA = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dq8_oracle.c")
_LIB = os.path.join(_HERE, "libdq8_oracle.so")
_CFLAGS = ["-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-Wextra"]
_lib = None


def build(force=False):
    """Compile dq8_oracle.c next to its source; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc"] + _CFLAGS + ["-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_sz, c_f, c_u8 = ctypes.c_size_t, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint8)
        lib.dq8o_codebook.argtypes = [ctypes.c_int, c_f]
        lib.dq8o_absmax.argtypes = [c_f, c_sz, c_sz, c_f]
        lib.dq8o_encode.argtypes = [ctypes.c_int, c_f, c_sz, c_sz, c_f, c_u8, ctypes.c_int]
        lib.dq8o_decode.argtypes = [ctypes.c_int, c_u8, c_f, c_sz, c_sz, c_f]
        lib.dq8o_decode_accumulate_avg.argtypes = [ctypes.c_int, ctypes.POINTER(c_u8), ctypes.POINTER(c_f),
                                                   ctypes.c_int, c_sz, c_sz, c_f]
        lib.dq8o_decode_accumulate_avg_local.argtypes = [ctypes.c_int, ctypes.POINTER(c_u8), ctypes.POINTER(c_f),
                                                         ctypes.c_int, c_f, c_sz, c_sz, c_f]
        lib.dq8o_decode_avg_encode.argtypes = [ctypes.c_int, ctypes.POINTER(c_u8), ctypes.POINTER(c_f), ctypes.c_int,
                                               c_f, c_sz, c_sz, c_f, c_u8]
        c_d = ctypes.POINTER(ctypes.c_double)
        lib.dq8o_error_stats.argtypes = [ctypes.c_int, c_f, c_sz, c_sz, c_f, ctypes.c_int, c_d, c_d]
        lib.dq8o_set_threads.argtypes = [ctypes.c_int]
        for f in (lib.dq8o_error_stats, lib.dq8o_codebook, lib.dq8o_absmax, lib.dq8o_encode, lib.dq8o_decode,
                  lib.dq8o_decode_accumulate_avg, lib.dq8o_decode_accumulate_avg_local, lib.dq8o_decode_avg_encode,
                  lib.dq8o_set_threads, lib.dq8o_get_threads):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _bp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s failed with status %d" % (what, rc))


def _f32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("expected float32, got %s" % a.dtype)
    return a.reshape(-1)


def _u8(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint8:
        raise TypeError("expected uint8, got %s" % a.dtype)
    return a.reshape(-1)


def _non_negative(scales):
    """A given scale stands for an absolute maximum or a power of ten (Sec. 3.1): finite, sign bit clear."""
    if np.any(np.signbit(scales)) or not np.all(np.isfinite(scales)):
        raise ValueError("given scales must be finite and >= 0 (sign bit clear)")


def n_blocks(n, block):
    if n == 0:
        return 0
    b = n if block == 0 else block
    return (n + b - 1) // b


def set_threads(t):
    """Threads used for the block loop (timing only; results do not depend on it)."""
    return _load().dq8o_set_threads(int(t))


def codebook(kind):
    cb = np.empty(256, dtype=np.float32)
    _check(_load().dq8o_codebook(int(kind), _fp(cb)), "codebook")
    return cb


def absmax(x, block=0):
    x = _f32(x)
    scales = np.empty(n_blocks(x.size, block), dtype=np.float32)
    _check(_load().dq8o_absmax(_fp(x), x.size, int(block), _fp(scales)), "absmax")
    return scales


def encode(kind, x, block=0, scales=None):
    """Returns (codes uint8[n], scales float32[nb]).  scales given -> used as input."""
    x = _f32(x)
    given = scales is not None
    if given:
        scales = _f32(scales).copy()
        if scales.size != n_blocks(x.size, block):
            raise ValueError("scales has %d entries, want %d" % (scales.size, n_blocks(x.size, block)))
        _non_negative(scales)
    else:
        scales = np.empty(n_blocks(x.size, block), dtype=np.float32)
    codes = np.empty(x.size, dtype=np.uint8)
    _check(_load().dq8o_encode(int(kind), _fp(x), x.size, int(block), _fp(scales), _bp(codes), int(given)),
           "encode")
    return codes, scales


def decode(kind, codes, scales, block=0):
    codes, scales = _u8(codes), _f32(scales)
    if scales.size != n_blocks(codes.size, block):
        raise ValueError("scales has %d entries, want %d" % (scales.size, n_blocks(codes.size, block)))
    out = np.empty(codes.size, dtype=np.float32)
    _check(_load().dq8o_decode(int(kind), _bp(codes), _fp(scales), codes.size, int(block), _fp(out)), "decode")
    return out


def _segments(n, bounds):
    b = np.asarray(bounds, dtype=np.int64)
    if b.ndim != 1 or b.size < 2 or b[0] != 0 or b[-1] != n or np.any(np.diff(b) < 0):
        raise ValueError("bounds must ascend from 0 to n")
    return b


def absmax_segments(x, bounds):
    """Sec. 3.1, last paragraph, for matrices laid out back to back: every segment [bounds[i], bounds[i + 1]) by
    itself with one scale (block 0); an empty segment has scale +0."""
    x = _f32(x)
    b = _segments(x.size, bounds)
    scales = np.zeros(b.size - 1, dtype=np.float32)
    for i in range(b.size - 1):
        if b[i + 1] > b[i]:
            scales[i] = absmax(x[b[i]:b[i + 1]], 0)[0]
    return scales


def encode_segments(kind, x, bounds, scales=None):
    """encode() of every segment by itself with one scale each.  Returns (codes, scales)."""
    x = _f32(x)
    b = _segments(x.size, bounds)
    given = scales is not None
    out_scales = _f32(scales).copy() if given else np.zeros(b.size - 1, dtype=np.float32)
    if out_scales.size != b.size - 1:
        raise ValueError("scales has %d entries, want %d" % (out_scales.size, b.size - 1))
    codes = np.empty(x.size, dtype=np.uint8)
    for i in range(b.size - 1):
        if b[i + 1] > b[i]:
            c, s = encode(kind, x[b[i]:b[i + 1]], 0, scales=out_scales[i:i + 1] if given else None)
            codes[b[i]:b[i + 1]] = c
            out_scales[i] = s[0]
    return codes, out_scales


def decode_segments(kind, codes, scales, bounds):
    """decode() of every segment by itself with its scale."""
    codes, scales = _u8(codes), _f32(scales)
    b = _segments(codes.size, bounds)
    if scales.size != b.size - 1:
        raise ValueError("scales has %d entries, want %d" % (scales.size, b.size - 1))
    out = np.empty(codes.size, dtype=np.float32)
    for i in range(b.size - 1):
        if b[i + 1] > b[i]:
            out[b[i]:b[i + 1]] = decode(kind, codes[b[i]:b[i + 1]], scales[i:i + 1], 0)
    return out


def decode_accumulate_avg_segments(kind, codes_list, scales_list, bounds, local=None):
    """decode_accumulate_avg() of every segment by itself, scales_list[k][i] = worker k's scale of segment i."""
    n = _f32(local).size if local is not None else _u8(codes_list[0]).size
    b = _segments(n, bounds)
    out = np.empty(n, dtype=np.float32)
    for i in range(b.size - 1):
        lo, hi = b[i], b[i + 1]
        if hi > lo:
            out[lo:hi] = decode_accumulate_avg(kind, [_u8(c)[lo:hi] for c in codes_list], [_f32(s)[i:i + 1] for s in scales_list], 0,
                                               local=None if local is None else _f32(local)[lo:hi])
    return out


def _workers(codes_list, scales_list, block, n=None):
    K = len(codes_list)
    if K != len(scales_list):
        raise ValueError("codes_list and scales_list differ in length")
    codes_list = [_u8(c) for c in codes_list]
    scales_list = [_f32(s) for s in scales_list]
    if n is None:
        n = codes_list[0].size if K else 0
    for c, s in zip(codes_list, scales_list):
        if c.size != n or s.size != n_blocks(n, block):
            raise ValueError("worker buffers differ in size")
    cp = (ctypes.POINTER(ctypes.c_uint8) * max(K, 1))(*[_bp(c) for c in codes_list])
    sp = (ctypes.POINTER(ctypes.c_float) * max(K, 1))(*[_fp(s) for s in scales_list])
    return K, n, cp, sp, (codes_list, scales_list)  # the last item keeps the arrays alive


def decode_accumulate_avg(kind, codes_list, scales_list, block=0, local=None):
    """Mean of the K decoded buffers; with ``local`` the fp32 array is the first of K + 1 terms."""
    if local is None:
        K, n, cp, sp, _keep = _workers(codes_list, scales_list, block)
        out = np.empty(n, dtype=np.float32)
        _check(_load().dq8o_decode_accumulate_avg(int(kind), cp, sp, K, n, int(block), _fp(out)),
               "decode_accumulate_avg")
        return out
    local = _f32(local)
    K, n, cp, sp, _keep = _workers(codes_list, scales_list, block, local.size)
    out = np.empty(n, dtype=np.float32)
    _check(_load().dq8o_decode_accumulate_avg_local(int(kind), cp, sp, K, _fp(local), n, int(block), _fp(out)),
           "decode_accumulate_avg_local")
    return out


def decode_avg_encode(kind, codes_list, scales_list, block=0, local=None):
    """Average (optionally with the fp32 ``local`` term) and compress the average: (codes, scales)."""
    if local is not None:
        local = _f32(local)
    K, n, cp, sp, _keep = _workers(codes_list, scales_list, block, None if local is None else local.size)
    out_codes = np.empty(n, dtype=np.uint8)
    out_scales = np.empty(n_blocks(n, block), dtype=np.float32)
    lp = _fp(local) if local is not None else ctypes.POINTER(ctypes.c_float)()
    _check(_load().dq8o_decode_avg_encode(int(kind), cp, sp, K, lp, n, int(block), _fp(out_scales), _bp(out_codes)),
           "decode_avg_encode")
    return out_codes, out_scales


def error_stats(kind, x, block=0, scales=None):
    """Approximation error of compress-then-decompress (Sec. 3.4, Table 2).

    Returns (stats float64[nb, 4], means float64[2]): per block the sum of absolute errors, the
    sum of relative errors over non-zero inputs, the number of non-zero inputs and the largest
    absolute error; means = (mean absolute error, mean relative error over non-zero inputs).
    scales given -> used instead of the absolute maxima."""
    x = _f32(x)
    given = scales is not None
    nb = n_blocks(x.size, block)
    if given:
        scales = _f32(scales).copy()
        if scales.size != nb:
            raise ValueError("scales has %d entries, want %d" % (scales.size, nb))
        _non_negative(scales)
    else:
        scales = np.empty(nb, dtype=np.float32)
    stats = np.zeros((nb, 4), dtype=np.float64)
    means = np.zeros(2, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    _check(_load().dq8o_error_stats(int(kind), _fp(x), x.size, int(block), _fp(scales), int(given),
                                    stats.ctypes.data_as(dp), means.ctypes.data_as(dp)), "error_stats")
    return stats, means
