"""Entry points of libdq8.so that are not part of the public ABI (csrc/dq8_internal.h), for the
benchmark's calibration and for launch-shape experiments.  Nothing here is needed to use the codec."""
import ctypes

from . import dq8


def _lib():
    L = dq8.lib()
    if not getattr(L, "_dq8_internal_bound", False):
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.dq8_internal_copy.argtypes = [vp, vp, sz, vp]
        L.dq8_internal_copy.restype = ci
        L.dq8_internal_tune.argtypes = [ctypes.c_char_p, ci]
        L.dq8_internal_tune.restype = ci
        L.dq8_internal_device_info.argtypes = [ctypes.POINTER(ci)]
        L.dq8_internal_device_info.restype = ci
        L._dq8_internal_bound = True
    return L


def calibration_copy(dst, src):
    """Plain fp32 device copy with the kernels' access pattern (bandwidth / counter calibration only)."""
    import torch
    src = dq8._dev(src, torch.float32, "src")
    dst = dq8._dev(dst, torch.float32, "dst")
    if dst.numel() < src.numel():
        raise ValueError("dst too small")
    with dq8._on(src.device):
        dq8._check(_lib().dq8_internal_copy(dst.data_ptr(), src.data_ptr(), src.numel(), dq8._stream()), "dq8_internal_copy")
    return dst


def tune(**kw):
    """Changes launch-shape parameters (only in a library built with -DDQ8_TUNABLE; results never depend on them)."""
    for k, v in kw.items():
        dq8._check(_lib().dq8_internal_tune(k.encode(), int(v)), "dq8_internal_tune(%s)" % k)


def device_info():
    """Compute units, peak clocks (MHz), memory bus width (bits) and L2 size (bytes) of the current device."""
    out = (ctypes.c_int * 5)()
    dq8._check(_lib().dq8_internal_device_info(out), "dq8_internal_device_info")
    return {"compute_units": out[0], "peak_engine_clock_MHz": out[1] / 1000.0, "peak_memory_clock_MHz": out[2] / 1000.0,
            "memory_bus_bits": out[3], "l2_bytes": out[4]}
