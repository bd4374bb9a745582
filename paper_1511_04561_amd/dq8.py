"""Python binding of the dq8 C ABI (include/dq8.h): argument marshalling only.

Every function takes torch CUDA tensors (device memory) and enqueues the library's
HIP kernels on torch's current stream.  Nothing is computed here and there is no
fallback: if libdq8.so is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

DYNAMIC_TREE, LINEAR, STATIC_TREE, MANTISSA = 0, 1, 2, 3
SCALES_GIVEN = 1
MAX_K = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
# DQ8_LIBRARY names another build of the same library (e.g. one compiled with -DDQ8_TUNABLE for experiments).
LIB_PATH = os.environ.get("DQ8_LIBRARY") or os.path.join(_HERE, "libdq8.so")
_lib = None


class Dq8Error(RuntimeError):
    pass


def lib():
    """The loaded shared library (loaded on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise Dq8Error("%s not found: build it with `python -m paper_1511_04561_amd.build` "
                           "(there is no fallback path)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.dq8_codebook.argtypes = [ci, vp]
        L.dq8_init.argtypes = []
        L.dq8_absmax.argtypes = [vp, sz, sz, vp, vp]
        L.dq8_encode.argtypes = [ci, vp, sz, sz, vp, vp, ctypes.c_uint, vp]
        L.dq8_decode.argtypes = [ci, vp, vp, sz, sz, vp, vp]
        L.dq8_decode_accumulate_avg.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, sz, sz, vp, vp]
        L.dq8_decode_accumulate_avg_local.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, sz, sz, vp, vp]
        L.dq8_decode_avg_encode.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, sz, sz, vp, vp, vp]
        L.dq8_error_stats.argtypes = [ci, vp, sz, sz, vp, ctypes.c_uint, vp, vp, vp]
        L.dq8_absmax_segments.argtypes = [vp, sz, vp, sz, vp, vp]
        L.dq8_encode_segments.argtypes = [ci, vp, sz, vp, sz, vp, vp, ctypes.c_uint, vp]
        L.dq8_decode_segments.argtypes = [ci, vp, vp, sz, vp, sz, vp, vp]
        L.dq8_decode_accumulate_avg_segments.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, sz, vp, sz, vp, vp]
        for f in (L.dq8_codebook, L.dq8_init, L.dq8_absmax, L.dq8_encode, L.dq8_decode, L.dq8_decode_accumulate_avg,
                  L.dq8_decode_accumulate_avg_local, L.dq8_decode_avg_encode, L.dq8_absmax_segments, L.dq8_encode_segments,
                  L.dq8_decode_segments, L.dq8_decode_accumulate_avg_segments):
            f.restype = ci
        dbl = ctypes.c_double
        L.dq8_model_speedup.argtypes = [ci, dbl, dbl, dbl, ci, dbl, dbl, ctypes.POINTER(dbl)]
        L.dq8_model_penalty.argtypes = [ctypes.POINTER(dbl), ctypes.POINTER(dbl), sz, ctypes.POINTER(dbl)]
        L.dq8_model_speedup.restype = ci
        L.dq8_model_penalty.restype = ci
        L.dq8_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise Dq8Error("%s failed (status %d): %s" % (what, rc, lib().dq8_last_error().decode()))


def n_blocks(n, block):
    if n == 0:
        return 0
    b = n if (block == 0 or block > n) else block
    return (n + b - 1) // b


def _dev(t, dtype, what):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA tensor" % what)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (what, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class _NoSwitch:
    def __enter__(self):
        return None

    def __exit__(self, *exc):
        return False


_NO_SWITCH = _NoSwitch()


def _on(device):
    """Makes `device` current for the call; nothing to do (and nothing spent) when it already is."""
    if device.index is None or device.index == torch.cuda.current_device():
        return _NO_SWITCH
    return torch.cuda.device(device)


def codebook(kind):
    """The 256 table values of a data type as a CPU float32 tensor."""
    cb = torch.empty(256, dtype=torch.float32)
    _check(lib().dq8_codebook(int(kind), cb.data_ptr()), "dq8_codebook")
    return cb


def init():
    _check(lib().dq8_init(), "dq8_init")


def absmax(x, block=0, scales=None):
    x = _dev(x, torch.float32, "x")
    n = x.numel()
    if scales is None:
        scales = torch.empty(n_blocks(n, block), dtype=torch.float32, device=x.device)
    _dev(scales, torch.float32, "scales")
    if scales.numel() < n_blocks(n, block):
        raise ValueError("scales too small")
    with _on(x.device):
        _check(lib().dq8_absmax(x.data_ptr(), n, int(block), scales.data_ptr(), _stream()), "dq8_absmax")
    return scales


def encode(kind, x, block=0, scales=None, codes=None, scales_given=False):
    """Returns (codes, scales).  With scales_given the passed scales are used as they are."""
    x = _dev(x, torch.float32, "x")
    n = x.numel()
    if scales is None:
        if scales_given:
            raise ValueError("scales_given needs scales")
        scales = torch.empty(n_blocks(n, block), dtype=torch.float32, device=x.device)
    if codes is None:
        codes = torch.empty(n, dtype=torch.uint8, device=x.device)
    _dev(scales, torch.float32, "scales")
    _dev(codes, torch.uint8, "codes")
    if scales.numel() < n_blocks(n, block) or codes.numel() < n:
        raise ValueError("output buffers too small")
    with _on(x.device):
        _check(lib().dq8_encode(int(kind), x.data_ptr(), n, int(block), scales.data_ptr(), codes.data_ptr(),
                                SCALES_GIVEN if scales_given else 0, _stream()), "dq8_encode")
    return codes, scales


def decode(kind, codes, scales, block=0, out=None):
    codes = _dev(codes, torch.uint8, "codes")
    scales = _dev(scales, torch.float32, "scales")
    n = codes.numel()
    if scales.numel() < n_blocks(n, block):
        raise ValueError("scales too small")
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "out")
    if out.numel() < n:
        raise ValueError("out too small")
    with _on(codes.device):
        _check(lib().dq8_decode(int(kind), codes.data_ptr(), scales.data_ptr(), n, int(block), out.data_ptr(),
                                _stream()), "dq8_decode")
    return out


MAX_SEGMENTS = 4095


def _bounds(bounds, n):
    """bounds: int64 device tensor of n_seg + 1 ascending element offsets from 0 to n (read by the kernels only)."""
    b = _dev(bounds, torch.int64, "bounds")
    if b.numel() < 2:
        raise ValueError("bounds needs at least two entries")
    return b, b.numel() - 1


def absmax_segments(x, bounds, scales=None):
    x = _dev(x, torch.float32, "x")
    b, n_seg = _bounds(bounds, x.numel())
    if scales is None:
        scales = torch.empty(n_seg, dtype=torch.float32, device=x.device)
    _dev(scales, torch.float32, "scales")
    if scales.numel() < n_seg:
        raise ValueError("scales too small")
    with _on(x.device):
        _check(lib().dq8_absmax_segments(x.data_ptr(), x.numel(), b.data_ptr(), n_seg, scales.data_ptr(), _stream()),
               "dq8_absmax_segments")
    return scales


def encode_segments(kind, x, bounds, scales=None, codes=None, scales_given=False):
    """Tensors back to back in x, one scale each.  Returns (codes, scales)."""
    x = _dev(x, torch.float32, "x")
    n = x.numel()
    b, n_seg = _bounds(bounds, n)
    if scales is None:
        if scales_given:
            raise ValueError("scales_given needs scales")
        scales = torch.empty(n_seg, dtype=torch.float32, device=x.device)
    if codes is None:
        codes = torch.empty(n, dtype=torch.uint8, device=x.device)
    _dev(scales, torch.float32, "scales")
    _dev(codes, torch.uint8, "codes")
    if scales.numel() < n_seg or codes.numel() < n:
        raise ValueError("output buffers too small")
    with _on(x.device):
        _check(lib().dq8_encode_segments(int(kind), x.data_ptr(), n, b.data_ptr(), n_seg, scales.data_ptr(), codes.data_ptr(),
                                         SCALES_GIVEN if scales_given else 0, _stream()), "dq8_encode_segments")
    return codes, scales


def decode_segments(kind, codes, scales, bounds, out=None):
    codes = _dev(codes, torch.uint8, "codes")
    scales = _dev(scales, torch.float32, "scales")
    n = codes.numel()
    b, n_seg = _bounds(bounds, n)
    if scales.numel() < n_seg:
        raise ValueError("scales too small")
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "out")
    if out.numel() < n:
        raise ValueError("out too small")
    with _on(codes.device):
        _check(lib().dq8_decode_segments(int(kind), codes.data_ptr(), scales.data_ptr(), n, b.data_ptr(), n_seg, out.data_ptr(),
                                         _stream()), "dq8_decode_segments")
    return out


def _workers(codes_list, scales_list, block, n=None):
    K = len(codes_list)
    if K != len(scales_list):
        raise ValueError("codes_list and scales_list differ in length")
    if n is None:
        if K == 0:
            raise ValueError("need at least one worker buffer")
        n = codes_list[0].numel()
    for c, s in zip(codes_list, scales_list):
        _dev(c, torch.uint8, "codes")
        _dev(s, torch.float32, "scales")
        if c.numel() != n or s.numel() < n_blocks(n, block):
            raise ValueError("worker buffers differ in size")
    cp = (ctypes.c_void_p * max(K, 1))(*[c.data_ptr() for c in codes_list])
    sp = (ctypes.c_void_p * max(K, 1))(*[s.data_ptr() for s in scales_list])
    return K, n, cp, sp


def decode_accumulate_avg(kind, codes_list, scales_list, block=0, out=None, local=None):
    """Mean of the K decoded buffers; with ``local`` (fp32) that array is the first of K + 1 terms."""
    if local is not None:
        _dev(local, torch.float32, "local")
    K, n, cp, sp = _workers(codes_list, scales_list, block, None if local is None else local.numel())
    dev = local.device if local is not None else codes_list[0].device
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=dev)
    _dev(out, torch.float32, "out")
    if out.numel() < n:
        raise ValueError("out too small")
    with _on(out.device):
        if local is None:
            _check(lib().dq8_decode_accumulate_avg(int(kind), cp, sp, K, n, int(block), out.data_ptr(), _stream()),
                   "dq8_decode_accumulate_avg")
        else:
            _check(lib().dq8_decode_accumulate_avg_local(int(kind), cp, sp, K, local.data_ptr(), n, int(block),
                                                         out.data_ptr(), _stream()), "dq8_decode_accumulate_avg_local")
    return out


def decode_accumulate_avg_segments(kind, codes_list, scales_list, bounds, out=None, local=None):
    """Mean of the K decoded buffers of tensors back to back, one scale per tensor and worker."""
    if local is not None:
        _dev(local, torch.float32, "local")
    K = len(codes_list)
    if K != len(scales_list) or (K == 0 and local is None):
        raise ValueError("need as many scale arrays as code arrays, and at least one worker or local")
    n = local.numel() if local is not None else codes_list[0].numel()
    b, n_seg = _bounds(bounds, n)
    for c, s in zip(codes_list, scales_list):
        _dev(c, torch.uint8, "codes")
        _dev(s, torch.float32, "scales")
        if c.numel() != n or s.numel() < n_seg:
            raise ValueError("worker buffers differ in size")
    cp = (ctypes.c_void_p * max(K, 1))(*[c.data_ptr() for c in codes_list])
    sp = (ctypes.c_void_p * max(K, 1))(*[s.data_ptr() for s in scales_list])
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=b.device)
    _dev(out, torch.float32, "out")
    if out.numel() < n:
        raise ValueError("out too small")
    with _on(out.device):
        _check(lib().dq8_decode_accumulate_avg_segments(int(kind), cp, sp, K, None if local is None else local.data_ptr(), n,
                                                        b.data_ptr(), n_seg, out.data_ptr(), _stream()),
               "dq8_decode_accumulate_avg_segments")
    return out


def decode_avg_encode(kind, codes_list, scales_list, block=0, local=None, scales=None, codes=None):
    """Average the K buffers (with ``local`` as first term if given) and compress the average: (codes, scales)."""
    if local is not None:
        _dev(local, torch.float32, "local")
    K, n, cp, sp = _workers(codes_list, scales_list, block, None if local is None else local.numel())
    dev = local.device if local is not None else codes_list[0].device
    if scales is None:
        scales = torch.empty(n_blocks(n, block), dtype=torch.float32, device=dev)
    if codes is None:
        codes = torch.empty(n, dtype=torch.uint8, device=dev)
    _dev(scales, torch.float32, "scales")
    _dev(codes, torch.uint8, "codes")
    if scales.numel() < n_blocks(n, block) or codes.numel() < n:
        raise ValueError("output buffers too small")
    with _on(codes.device):
        _check(lib().dq8_decode_avg_encode(int(kind), cp, sp, K, None if local is None else local.data_ptr(), n,
                                           int(block), scales.data_ptr(), codes.data_ptr(), _stream()),
               "dq8_decode_avg_encode")
    return codes, scales


def error_stats(kind, x, block=0, scales=None, scales_given=False, stats=None, means=None):
    """Approximation error of compress-then-decompress (Sec. 3.4, Table 2).

    Returns (stats float64[nb, 4], means float64[2]) on the device: per block the sum of absolute errors,
    the sum of relative errors over non-zero inputs, the number of non-zero inputs and the largest absolute
    error; means = (mean absolute error, mean relative error over non-zero inputs)."""
    x = _dev(x, torch.float32, "x")
    n = x.numel()
    nb = n_blocks(n, block)
    if scales is None:
        if scales_given:
            raise ValueError("scales_given needs scales")
        scales = torch.empty(nb, dtype=torch.float32, device=x.device)
    if stats is None:
        stats = torch.zeros((nb, 4), dtype=torch.float64, device=x.device)
    if means is None:
        means = torch.zeros(2, dtype=torch.float64, device=x.device)
    _dev(scales, torch.float32, "scales")
    _dev(stats, torch.float64, "stats")
    _dev(means, torch.float64, "means")
    if scales.numel() < nb or stats.numel() < 4 * nb or means.numel() < 2:
        raise ValueError("output buffers too small")
    with _on(x.device):
        _check(lib().dq8_error_stats(int(kind), x.data_ptr(), n, int(block), scales.data_ptr(),
                                     SCALES_GIVEN if scales_given else 0, stats.data_ptr(), means.data_ptr(), _stream()),
               "dq8_error_stats")
    return stats, means


def model_speedup(n_gpus, total_ms, fc_ms, conv_penalty_ms, sub_batches, parallel_fc_ms, fc_penalty_ms):
    """Predicted speed-up of the single-node model (host arithmetic in the library)."""
    out = ctypes.c_double()
    _check(lib().dq8_model_speedup(int(n_gpus), total_ms, fc_ms, conv_penalty_ms, int(sub_batches), parallel_fc_ms,
                                   fc_penalty_ms, ctypes.byref(out)), "dq8_model_speedup")
    return out.value


def model_penalty(transfer_ms, compute_ms):
    """Sum of the parts of the transfers that their overlapping computations do not cover."""
    n = len(transfer_ms)
    if n != len(compute_ms):
        raise ValueError("transfer_ms and compute_ms differ in length")
    arr = ctypes.c_double * max(n, 1)
    out = ctypes.c_double()
    _check(lib().dq8_model_penalty(arr(*transfer_ms), arr(*compute_ms), n, ctypes.byref(out)), "dq8_model_penalty")
    return out.value
