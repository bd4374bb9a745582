"""CPU-only tests of the HIP library's host side: it loads, exports the declared ABI, rejects
bad arguments without touching a device, and its tables / code search agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_1511_04561_amd import build as dq8_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KINDS = [0, 1, 2, 3]


@pytest.fixture(scope="module")
def L():
    dq8_build.build(force=False)  # compiles only when the library is missing or stale
    lib = ctypes.CDLL(dq8_build.LIB)
    lib.dq8_last_error.restype = ctypes.c_char_p
    return lib


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "dq8.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(dq8_[a-z0-9_]+)\s*\(", header)))
    assert names == ["dq8_absmax", "dq8_absmax_segments", "dq8_codebook", "dq8_decode", "dq8_decode_accumulate_avg",
                     "dq8_decode_accumulate_avg_local", "dq8_decode_accumulate_avg_segments", "dq8_decode_avg_encode", "dq8_decode_segments", "dq8_encode",
                     "dq8_encode_segments", "dq8_error_stats", "dq8_init",
                     "dq8_last_error", "dq8_model_penalty", "dq8_model_speedup"]
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("kind", KINDS)
def test_codebook_is_bit_identical_to_the_oracle(L, kind):
    cb = np.empty(256, np.float32)
    assert L.dq8_codebook(kind, cb.ctypes.data_as(ctypes.c_void_p)) == 0
    assert cb.tobytes() == oracle.codebook(kind).tobytes()


def test_argument_errors_need_no_device(L):
    buf = np.zeros(64, np.float32)
    p = buf.ctypes.data_as(ctypes.c_void_p)
    n = ctypes.c_size_t(16)
    z = ctypes.c_size_t(0)
    assert L.dq8_codebook(7, p) == 2 and b"7" in L.dq8_last_error()
    assert L.dq8_codebook(0, None) == 1
    assert L.dq8_absmax(None, n, z, p, None) == 1
    assert L.dq8_absmax(None, z, z, None, None) == 0  # n == 0 is a no-op
    assert L.dq8_encode(9, p, n, z, p, p, 0, None) == 2
    assert L.dq8_encode(0, p, n, z, p, p, 4, None) == 3  # unknown flag
    assert L.dq8_encode(0, None, n, z, p, p, 0, None) == 1
    assert L.dq8_encode(0, None, z, z, None, None, 0, None) == 0
    assert L.dq8_decode(-1, p, p, n, z, p, None) == 2
    assert L.dq8_decode(0, p, None, n, z, p, None) == 1
    assert L.dq8_decode(0, None, None, z, z, None, None) == 0
    # tensors back to back: the same checks, and the number of segments
    one, many = ctypes.c_size_t(1), ctypes.c_size_t(4096)
    q = np.zeros(64, np.float32).ctypes.data_as(ctypes.c_void_p)
    r = np.zeros(64, np.uint8).ctypes.data_as(ctypes.c_void_p)
    b = np.zeros(8, np.uint64).ctypes.data_as(ctypes.c_void_p)
    assert L.dq8_absmax_segments(None, n, b, one, q, None) == 1
    assert L.dq8_absmax_segments(p, n, None, one, q, None) == 1
    assert L.dq8_absmax_segments(p, n, b, z, q, None) == 3 and b"segments" in L.dq8_last_error()
    assert L.dq8_absmax_segments(p, n, b, many, q, None) == 3
    assert L.dq8_absmax_segments(None, z, None, z, None, None) == 0
    assert L.dq8_encode_segments(9, p, n, b, one, q, r, 0, None) == 2
    assert L.dq8_encode_segments(0, p, n, b, one, q, r, 2, None) == 3  # unknown flag
    assert L.dq8_encode_segments(0, p, n, b, one, p, r, 0, None) == 3 and b"overlap" in L.dq8_last_error()
    assert L.dq8_encode_segments(0, p, n, b, many, q, r, 0, None) == 3
    assert L.dq8_decode_segments(4, r, q, n, b, one, p, None) == 2
    assert L.dq8_decode_segments(0, r, q, n, None, one, p, None) == 1
    assert L.dq8_decode_segments(0, r, p, n, b, one, p, None) == 3  # out overlaps the scales
    assert L.dq8_decode_segments(0, None, None, z, None, z, None, None) == 0
    two = (ctypes.c_void_p * 2)(r, r)
    twos = (ctypes.c_void_p * 2)(q, q)
    assert L.dq8_decode_accumulate_avg_segments(0, two, twos, 0, None, n, b, one, p, None) == 3  # no worker and no local
    assert L.dq8_decode_accumulate_avg_segments(0, two, twos, 33, None, n, b, one, p, None) == 3
    assert L.dq8_decode_accumulate_avg_segments(0, two, twos, 2, None, n, None, one, p, None) == 1
    assert L.dq8_decode_accumulate_avg_segments(0, two, twos, 2, None, n, b, one, q, None) == 3  # out overlaps a worker's scales
    assert L.dq8_decode_accumulate_avg_segments(0, two, twos, 2, None, z, None, z, None, None) == 0
    arr = (ctypes.c_void_p * 2)(p, p)
    assert L.dq8_decode_accumulate_avg(0, arr, arr, 0, n, z, p, None) == 3
    assert L.dq8_decode_accumulate_avg(0, arr, arr, 33, n, z, p, None) == 3
    assert L.dq8_decode_accumulate_avg(0, None, arr, 2, n, z, p, None) == 1
    assert L.dq8_decode_accumulate_avg(5, arr, arr, 2, n, z, p, None) == 2
    assert L.dq8_decode_accumulate_avg(0, arr, arr, 2, z, z, None, None) == 0
    # the average with a local term and the average-then-compress round
    assert L.dq8_decode_accumulate_avg_local(0, arr, arr, -1, p, n, z, p, None) == 3
    assert L.dq8_decode_accumulate_avg_local(0, arr, arr, 33, p, n, z, p, None) == 3
    assert L.dq8_decode_accumulate_avg_local(0, arr, arr, 2, None, n, z, p, None) == 1
    assert L.dq8_decode_accumulate_avg_local(4, arr, arr, 2, p, n, z, p, None) == 2
    assert L.dq8_decode_accumulate_avg_local(0, arr, arr, 2, p, n, z, p, None) == 3  # out overlaps local
    assert L.dq8_decode_accumulate_avg_local(0, None, None, 0, None, z, z, None, None) == 0
    assert L.dq8_decode_avg_encode(0, arr, arr, 0, None, n, z, p, p, None) == 3  # no worker and no local term
    assert L.dq8_decode_avg_encode(0, arr, arr, 2, None, n, z, None, p, None) == 1
    assert L.dq8_decode_avg_encode(4, arr, arr, 2, None, n, z, p, p, None) == 2
    big = ctypes.c_size_t(40000)
    assert L.dq8_decode_avg_encode(0, arr, arr, 2, None, big, z, p, p, None) == 3  # one block of 40000 > 16384
    assert b"16384" in L.dq8_last_error()
    assert L.dq8_decode_avg_encode(0, arr, arr, 2, None, big, ctypes.c_size_t(20000), p, p, None) == 3
    assert b"16384" in L.dq8_last_error()
    assert L.dq8_decode_avg_encode(0, arr, arr, 2, None, n, z, p, p, None) == 3  # outputs overlap each other
    assert L.dq8_decode_avg_encode(0, arr, arr, 2, None, z, z, None, None, None) == 0
    # approximation-error statistics
    assert L.dq8_error_stats(9, p, n, z, p, 0, p, None, None) == 2
    assert L.dq8_error_stats(0, p, n, z, p, 2, p, None, None) == 3   # unknown flag
    assert L.dq8_error_stats(0, None, n, z, p, 0, p, None, None) == 1
    assert L.dq8_error_stats(0, p, n, z, p, 0, None, None, None) == 1
    assert L.dq8_error_stats(0, p, n, z, p, 0, p, None, None) == 3   # x, scales and stats are one buffer
    assert L.dq8_error_stats(0, None, z, z, None, 0, None, None, None) == 0
    assert isinstance(L.dq8_last_error(), bytes)


def _tables(L, kind):
    cb, thr = np.empty(256, np.float32), np.empty(127, np.float32)
    lo, nbk = ctypes.c_uint32(), ctypes.c_uint32()
    bucket = np.empty(4096, np.uint32)
    rc = L.dq8_internal_tables(kind, cb.ctypes.data_as(ctypes.c_void_p), thr.ctypes.data_as(ctypes.c_void_p),
                               ctypes.byref(lo), ctypes.byref(nbk), bucket.ctypes.data_as(ctypes.c_void_p), 4096)
    assert rc == 0
    return cb, thr, lo.value, nbk.value, bucket[:nbk.value]


def _ranks(L, kind):
    n_mag, canon = ctypes.c_uint32(), np.empty(128, np.uint8)
    assert L.dq8_internal_ranks(kind, ctypes.byref(n_mag), canon.ctypes.data_as(ctypes.c_void_p)) == 0
    return n_mag.value, canon


def _distinct_magnitudes(kind):
    """Ascending distinct magnitudes of the oracle's table and the smallest field of each."""
    o = oracle.codebook(kind)[:128]
    vals, first = np.unique(o, return_index=True)  # first occurrence = smallest field
    return vals, first


@pytest.mark.parametrize("kind", KINDS)
def test_ranks_are_the_distinct_magnitudes_with_their_smallest_field(L, kind):
    n_mag, canon = _ranks(L, kind)
    vals, first = _distinct_magnitudes(kind)
    assert n_mag == vals.size
    assert np.array_equal(canon[:n_mag], first.astype(np.uint8))
    assert np.all(canon[n_mag:] == canon[n_mag - 1])
    if kind != 3:
        assert n_mag == 128 and np.array_equal(canon, np.arange(128, dtype=np.uint8))
    else:  # the 8 zeros count once, and m = 10 of decades 0..6 repeats m = 1 of the next
        assert n_mag == 128 - 7 - 7


@pytest.mark.parametrize("kind", KINDS)
def test_thresholds_are_the_first_binary32_above_each_midpoint(L, kind):
    cb, thr, lo, nbk, bucket = _tables(L, kind)
    vals, _ = _distinct_magnitudes(kind)
    o = vals.astype(np.float64)
    n_thr = o.size - 1
    mid = (o[:-1] + o[1:]) / 2
    assert np.all(np.isinf(thr[n_thr:]))
    thr = thr[:n_thr]
    t = thr.astype(np.float64)
    below = np.nextafter(thr, np.float32(0)).astype(np.float64)
    assert np.all(t > mid) and np.all(below <= mid)
    hi = lo + nbk - 1  # first and last bucket hold no threshold
    tb = thr.view(np.uint32)
    # (the table is built from the thresholds moved down by the proximity window of 4 binary32 steps)
    assert nbk <= 4352 - 260 and ((int(tb[0]) - 4) >> 16) == lo + 1 and ((int(tb[-1]) + 4) >> 16) == hi - 1 and hi <= 0x3FC0


@pytest.mark.parametrize("kind", KINDS)
def test_code_search_equals_threshold_count_for_every_binary32_value(L, kind):
    bad, missed = ctypes.c_uint64(123), ctypes.c_uint64(123)
    assert L.dq8_internal_check_search(kind, ctypes.byref(bad), ctypes.byref(missed)) == 0
    assert bad.value == 0      # the flattened search is the threshold count, for every bit pattern
    assert missed.value == 0   # and every value next to a threshold raises the proximity flag


def _encode_host(L, kind, x, scale, use_reciprocal):
    L.dq8_internal_encode_host.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_void_p]
    x = np.ascontiguousarray(x, np.float32)
    got = np.empty(x.size, np.uint8)
    n_exact = ctypes.c_uint64()
    assert L.dq8_internal_encode_host(kind, x.ctypes.data_as(ctypes.c_void_p), x.size, float(scale), int(use_reciprocal),
                                      got.ctypes.data_as(ctypes.c_void_p), ctypes.byref(n_exact)) == 0
    return got, n_exact.value


@pytest.mark.parametrize("kind", KINDS)
def test_code_search_equals_the_oracle_on_normalised_values(L, kind):
    rng = np.random.Generator(np.random.PCG64(77))
    cb = _distinct_magnitudes(kind)[0]
    mid = ((cb[:-1].astype(np.float64) + cb[1:]) / 2).astype(np.float32).view(np.int32).astype(np.int64)
    near = (mid[:, None] + np.arange(-40, 41)[None, :]).reshape(-1).astype(np.int32).view(np.float32)
    pos = np.concatenate([near, rng.random(300000).astype(np.float32),
                          np.exp(rng.uniform(-25, 0, 300000)).astype(np.float32), np.array([0, 1, 2.5], np.float32)])
    x = np.concatenate([pos, -pos])
    want, _ = oracle.encode(kind, x, 0, scales=np.ones(1, np.float32))
    for recip in (0, 1):
        got, _ = _encode_host(L, kind, x, 1.0, recip)
        assert np.array_equal(got, want)


def test_reciprocal_product_is_within_three_steps_of_the_quotient():
    """The encoder's shortcut rests on |bits(x * fl(1/s)) - bits(fl(x / s))| <= 3 for normal results."""
    rng = np.random.Generator(np.random.PCG64(78))
    worst = 0
    for rep in range(8):
        n = 1 << 21
        s = np.exp(rng.uniform(-60, 60, n)).astype(np.float32)
        x = (s * rng.uniform(2.0 ** -27, 1.0, n)).astype(np.float32)
        if rep % 2:  # mantissas at the edges of a binade are the worst case
            s = (s.view(np.uint32) | np.uint32(0x7FFFF0)).view(np.float32) if rep % 4 == 1 else \
                (s.view(np.uint32) & np.uint32(0xFF80000F)).view(np.float32)
        r = (np.float32(1.0) / s).astype(np.float32)
        q0 = (x * r).astype(np.float32)
        q = (x / s).astype(np.float32)
        d = np.abs(q0.view(np.int32).astype(np.int64) - q.view(np.int32).astype(np.int64))
        worst = max(worst, int(d.max()))
    assert worst <= 3, worst


def test_division_by_a_power_of_two_equals_the_product_with_its_reciprocal():
    """The K-way average multiplies by 1/K when K is a power of two: bit-identical to the division,
    also where the result is subnormal, zero (either sign) or the sum is huge."""
    rng = np.random.Generator(np.random.PCG64(79))
    bits = rng.integers(0, 1 << 32, 1 << 22, dtype=np.uint64).astype(np.uint32)
    a = bits.view(np.float32)
    a = a[np.isfinite(a)]
    edge = np.array([0.0, -0.0, 2.0 ** -149, -2.0 ** -149, 3 * 2.0 ** -149, 2.0 ** -126, 1.5 * 2.0 ** -126,
                     np.finfo(np.float32).max, -np.finfo(np.float32).max], dtype=np.float32)
    small = (rng.integers(-(1 << 24), 1 << 24, 1 << 16).astype(np.float64) * 2.0 ** -149).astype(np.float32)
    a = np.concatenate([a, edge, small])
    for K in (1, 2, 4, 8, 16, 32):
        q = (a / np.float32(K)).astype(np.float32)
        m = (a * (np.float32(1.0) / np.float32(K))).astype(np.float32)
        assert np.array_equal(q.view(np.uint32), m.view(np.uint32)), K


def test_division_by_any_other_worker_count_in_three_instructions(tmp_path):
    """A number of terms that is not a power of two: the kernels form a * fl(1/count), its exact remainder and one
    correction instead of the division (csrc/dq8_arith.hpp).  The same function, compiled for the host, equals the
    correctly rounded quotient for every significand, both signs, every count 3 .. 33 and binades across the range
    that the kernels' test of the scales allows."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("needs g++")
    exe = str(tmp_path / "division_main")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "paper_1511_04561_amd", "csrc"), "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize", "division_main.cpp"), "-o", exe])
    p = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert p.returncode == 0 and "division checks ok" in p.stdout, p.stdout[-2000:]


@pytest.mark.parametrize("kind", KINDS)
def test_reciprocal_path_matches_the_oracle_around_every_threshold(L, kind):
    """Inputs built so that x / s lands on, and next to, every decision point, for awkward scales."""
    cb = _distinct_magnitudes(kind)[0]
    mid = ((cb[:-1].astype(np.float64) + cb[1:]) / 2)
    rng = np.random.Generator(np.random.PCG64(79 + kind))
    total_exact = 0
    for s in [1.0, 3.0, 0.7310585975646973, 1e-3, 1.9999998807907104, 1.0000001192092896, 5e-20, 7e19, 2.0 ** -100,
              2.0 ** 100, 1e-38, 3e38, 1.1e-30]:
        s32 = np.float32(s)
        with np.errstate(over="ignore"):  # products beyond binary32 become inf and are dropped below
            base = (mid * float(s32)).astype(np.float32).view(np.int32).astype(np.int64)
        x = (base[:, None] + np.arange(-12, 13)[None, :]).reshape(-1)
        x = x[(x > 0) & (x < 0x7F800000)].astype(np.int32).view(np.float32)
        x = x[np.abs(x) <= s32]
        extra = (rng.random(20000) * float(s32)).astype(np.float32)
        x = np.concatenate([x, -x, extra, -extra, np.array([s32, -s32, 0.0, -0.0], np.float32)])
        want, _ = oracle.encode(kind, x, 0, scales=np.array([s32], np.float32))
        got, n_exact = _encode_host(L, kind, x, s32, 1)
        assert np.array_equal(got, want), s
        got0, n_all = _encode_host(L, kind, x, s32, 0)
        assert np.array_equal(got0, want) and n_all == x.size
        total_exact += n_exact
    assert total_exact > 0  # the fallback was exercised


def test_launch_plan_covers_every_element_once(L):
    L.dq8_internal_plan.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                    ctypes.c_void_p]
    out = (ctypes.c_size_t * 6)()
    for n, block in [(61100840, 4096), (61100840, 0), (1, 0), (4097, 4096), (100, 7), (10 ** 6, 6000), (5000, 10 ** 9),
                     (4096 * 5000, 8192), (12345, 1)]:
        for wpc, wpb, unit in [(8, 1, 4096), (16, 1, 1024), (8, 4, 4096), (3, 4, 4096), (8, 1, 256)]:
            assert L.dq8_internal_plan(n, block, 256, wpc, wpb, unit, out) == 0
            B, nb, upb, units, teams, grid = list(out)
            Bw = n if (block == 0 or block > n) else block
            assert B == Bw and nb == (n + Bw - 1) // Bw and upb == (Bw + unit - 1) // unit
            full, last = divmod(n, Bw)
            assert units == full * upb + (last + unit - 1) // unit
            assert teams == grid * (4 // wpb) and grid >= 1 and teams <= max(1, 256 * wpc // wpb) + 3
            per_team = -(-units // teams)
            assert (per_team - 1) * teams < units  # balanced: no team walks more than one unit more than another
    assert L.dq8_internal_plan(10, 0, 256, 8, 3, 4096, out) == 3
    assert L.dq8_internal_plan(10, 0, 256, 8, 1, 1000, out) == 3


def test_the_shipped_library_has_fixed_launch_shapes(L):
    """Launch shapes are constants of the shipped build (nothing mutable is shared between threads); only a build
    with -DDQ8_TUNABLE accepts changes."""
    assert L.dq8_internal_tune(b"enc_wpc", 8) == 3 and b"DQ8_TUNABLE" in L.dq8_last_error()
    assert L.dq8_internal_tune(None, 8) == 1
    import paper_1511_04561_amd.dq8 as binding
    assert not hasattr(binding, "tune") and not hasattr(binding, "calibration_copy")


def test_units_follow_the_block_length(L):
    """Units of the piecewise kernels are no longer than a block (and the wavefronts per compute unit grow as
    they shrink); the kernels that hold a block take the smallest power of two that holds it, up to 4096."""
    def units(n, block, quads=16, wpc=4):
        out = (ctypes.c_size_t * 4)()
        assert L.dq8_internal_units(ctypes.c_size_t(n), ctypes.c_size_t(block), quads, wpc, out) == 0
        return list(out)
    n = 1 << 20
    assert units(n, 0) == [n, 4096, 4, 4096]            # one scale for the array
    assert units(n, 2 * n) == [n, 4096, 4, 4096]        # a block longer than the array is the array
    assert units(n, 4096) == [4096, 4096, 4, 4096]
    assert units(n, 4095) == [4095, 2048, 8, 4096]
    assert units(n, 3000) == [3000, 2048, 8, 4096]
    assert units(n, 2048) == [2048, 2048, 8, 2048]
    assert units(n, 1025) == [1025, 1024, 16, 2048]
    assert units(n, 1000) == [1000, 512, 32, 1024]
    assert units(n, 256) == [256, 256, 32, 256]
    assert units(n, 100) == [100, 256, 32, 256]          # never below one quad per lane
    assert units(n, 1) == [1, 256, 32, 256]
    assert units(n, 100000) == [100000, 4096, 4, 4096]
    assert units(n, 1000, quads=2, wpc=32) == [1000, 512, 32, 1024]
    assert units(100, 0) == [100, 256, 32, 256]
    assert L.dq8_internal_units(ctypes.c_size_t(n), ctypes.c_size_t(0), 3, 4, (ctypes.c_size_t * 4)()) == 3


def test_chunk_sizes_leave_few_empty_places(L):
    """Workers are averaged a chunk at a time: the chunk size wastes at most one place in eight and is as
    large as possible among the sizes that waste least."""
    got = {K: L.dq8_internal_chunk_size(K) for K in range(0, 33)}
    assert got[0] == 1 and got[1] == 1 and got[2] == 2
    for K in range(3, 33):
        c = got[K]
        assert 3 <= c <= 8
        waste = -K % c
        assert all(waste <= (-K % d) for d in range(3, 9)), (K, c)
        assert all(d <= c for d in range(3, 9) if (-K % d) == waste), (K, c)
    assert [got[K] for K in (3, 4, 5, 6, 7, 8, 10, 16, 24, 32)] == [3, 4, 5, 6, 7, 8, 5, 8, 8, 8]
