"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

Codes and scales are compared byte for byte; decoded and averaged fp32 values are compared
as raw bit patterns (0 ulp, -0 differs from +0).  Every input comes from the seeded
generators or from the oracle's own outputs, never from the HIP path.
"""
import os

import numpy as np
import pytest

import oracle
from paper_1511_04561_amd import workloads

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

KINDS = [0, 1, 2, 3]
NAMES = {0: "dynamic_tree", 1: "linear", 2: "static_tree", 3: "mantissa"}


@pytest.fixture(scope="module")
def dq8():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (select them with -m gpu on a GPU box)")
    from paper_1511_04561_amd import dq8 as mod
    mod.lib()  # a missing library is an error, not a skip
    mod.init()
    oracle.set_threads(16)
    return mod


PAD = 8192  # guard elements on both sides of every device array: two whole units

POISON = {np.dtype(np.float32): 3.0e38, np.dtype(np.uint8): 0xA5}


class Guarded:
    """A device array placed inside a larger buffer whose margins hold a known pattern.

    Inputs: a read past either end picks up the pattern (3e38 as a value, 0xA5 as a code), which
    changes scales or outputs.  Outputs: check() fails if a margin was written.
    `offset` shifts the first element by that many elements from an aligned address.
    """

    def __init__(self, n, dtype, offset=0, data=None):
        self.fill = POISON[np.dtype(dtype)]
        tdt = torch.float32 if np.dtype(dtype) == np.float32 else torch.uint8
        self.buf = torch.full((PAD + offset + n + PAD,), self.fill, dtype=tdt, device="cuda")
        self.lo, self.hi = PAD + offset, PAD + offset + n
        self.t = self.buf[self.lo:self.hi]
        if data is not None:
            self.t.copy_(torch.from_numpy(np.ascontiguousarray(data)))
        assert self.t.data_ptr() == self.buf.data_ptr() + self.lo * self.buf.element_size()

    def check(self, what):
        ok = bool((self.buf[:self.lo] == self.fill).all().item()) and bool((self.buf[self.hi:] == self.fill).all().item())
        assert ok, "%s: the kernel wrote outside its output array" % what


def dev(a, offset=0):
    """Guarded device copy of a numpy array (see Guarded)."""
    return Guarded(a.size, a.dtype, offset, a).t


def same_bits(got, want, what):
    got = got.cpu().numpy() if hasattr(got, "cpu") else got
    assert got.dtype == want.dtype and got.shape == want.shape, (what, got.dtype, got.shape, want.shape)
    if got.tobytes() != want.tobytes():
        word = {1: np.uint8, 4: np.uint32, 8: np.uint64}[got.dtype.itemsize]
        gi, wi = got.view(word), want.view(word)
        bad = np.nonzero(gi != wi)[0]
        raise AssertionError("%s: %d of %d differ, first at %d: got %r want %r" % (
            what, bad.size, got.size, bad[0], got[bad[0]], want[bad[0]]))


def check_encode_decode(dq8, kind, x, block, x_off=0, c_off=0, tag=""):
    print("case %s kind=%d n=%d block=%d x_off=%d c_off=%d" % (tag, kind, x.size, block, x_off, c_off), flush=True)
    want_codes, want_scales = oracle.encode(kind, x, block)
    want_out = oracle.decode(kind, want_codes, want_scales, block)
    nb = want_scales.size
    xd = dev(x, x_off)
    gc, gs = Guarded(x.size, np.uint8, c_off), Guarded(nb, np.float32)
    codes, scales = dq8.encode(kind, xd, block, scales=gs.t, codes=gc.t)
    same_bits(scales, want_scales, "scales " + tag)
    same_bits(codes, want_codes, "codes " + tag)
    gc.check("encode codes " + tag)
    gs.check("encode scales " + tag)
    ga = Guarded(nb, np.float32)
    same_bits(dq8.absmax(xd, block, scales=ga.t), want_scales, "absmax " + tag)
    ga.check("absmax " + tag)
    # encode with the scales handed in goes through the non-fused kernel
    gc2 = Guarded(x.size, np.uint8, c_off)
    codes2, _ = dq8.encode(kind, xd, block, scales=dev(want_scales), codes=gc2.t, scales_given=True)
    same_bits(codes2, want_codes, "codes(scales given) " + tag)
    gc2.check("encode(scales given) " + tag)
    # decode takes the oracle's codes as input
    go = Guarded(x.size, np.float32, x_off)
    out = dq8.decode(kind, dev(want_codes, c_off), dev(want_scales), block, out=go.t)
    same_bits(out, want_out, "decode " + tag)
    go.check("decode " + tag)


SHAPES = [  # (n, block)
    (3 * 4096 + 808, 4096),   # whole units and a ragged last block
    (4096, 4096), (4095, 4096), (4097, 4096), (1, 0), (3, 0), (5, 2), (63, 64), (65, 64),
    (100003, 0),              # one scale for the array, many units, tail not a multiple of 4
    (50 * 1000, 1000),        # rows shorter than a unit
    (7 * 6000 + 17, 6000),    # blocks of one full unit plus a partial one
    (5 * 8192 + 100, 8192),   # two units per block
    (1000, 7), (257, 1), (4096 * 3 + 1, 1),  # tiny blocks; the last wavefront's first unit is the ragged one
    (20000, 10 ** 9),         # block larger than the array
    (100 * 64 + 20, 64), (50 * 256 + 8, 256), (7 * 1024 + 4, 1024), (9 * 516 + 2, 516),  # short aligned blocks:
    (3 * 12000 + 40, 12000),  # whole quads, partly with a tail; a block of two whole units and a short aligned one
    # blocks of 4 .. 128 elements: many blocks per wavefront for the whole 1024-element units, the rest as above
    (5 * 1024 + 300, 64), (3 * 1024, 4), (2 * 1024 + 8, 8), (4 * 1024 + 100, 16), (7 * 1024 + 96, 32),
    (3 * 1024 + 640, 128), (40 * 1024 + 64, 64), (1024, 64), (1023, 64), (1025, 128), (9 * 512 + 100, 512),
    (6 * 1024 + 24, 1024),
    # blocks of 4097 .. 16384 elements are held by a team in units of 8192 / 16384 elements
    (3 * 16384 + 5000, 16384), (2 * 9216 + 4, 9216), (3 * 4100, 4100), (2 * 8196 + 3, 8196), (16384, 0),
    (2 * 8191, 8191), (2 * 16385, 16385), (4 * 8192, 8192), (5 * 12288, 12288),
    (5 * 2048 + 8, 2048), (4 * 3000, 3000), (3 * 2000 + 4, 2000), (2 * 3072 + 100, 3072), (3 * 1540, 1540),  # and in 2 or 3
    # blocks of whole quads that are not whole units: decompression walks units by position, up to 8 blocks per unit
    (500 * 40 + 3, 40), (300 * 100, 100), (70 * 200 + 1, 200), (900 * 36 + 2, 36), (33 * 588 + 7, 588), (40 * 340, 340),
    # compression of blocks of whole quads up to 1024 elements: a wavefront per block, with and without a short last block
    (500 * 40 + 4, 40), (64 * 200 + 8, 200), (9 * 1024 + 12, 1024), (100 * 12, 12), (21 * 600, 600), (2000 * 8, 8),
    (3 * 132, 132), (1000 * 260 + 256, 260),
]


@pytest.mark.parametrize("kind", KINDS)
def test_shapes_blocks_and_tails(dq8, kind):
    for i, (n, block) in enumerate(SHAPES):
        x = workloads.edge_case_block("wide", n, seed=1000 * kind + i)
        check_encode_decode(dq8, kind, x, block, tag="shape%d" % i)


@pytest.mark.parametrize("kind", KINDS)
def test_misaligned_pointers(dq8, kind):
    n = 2 * 4096 + 100
    x = workloads.edge_case_block("wide", n, seed=50 + kind)
    for x_off, c_off in [(1, 0), (0, 1), (3, 2), (2, 3)]:
        check_encode_decode(dq8, kind, x, 4096, x_off=x_off, c_off=c_off, tag="misaligned")
    x = workloads.edge_case_block("wide", 2 * 9216 + 100, seed=60 + kind)  # blocks held in a 16384-element unit
    for x_off, c_off in [(1, 0), (0, 2)]:
        check_encode_decode(dq8, kind, x, 9216, x_off=x_off, c_off=c_off, tag="misaligned-long")
        check_encode_decode(dq8, kind, x, 0, x_off=x_off, c_off=c_off, tag="misaligned-pertensor")


@pytest.mark.parametrize("kind", KINDS)
def test_degenerate_blocks(dq8, kind):
    B = 4096
    parts = [workloads.edge_case_block(c, B, seed=kind) for c in
             ("zeros", "neg_zeros", "denormal_absmax", "single_nonzero", "huge", "tiny", "wide")]
    parts.append(np.array([0.0, -0.0, 1e-45, -1e-45], np.float32))
    x = np.concatenate(parts)
    check_encode_decode(dq8, kind, x, B, tag="degenerate")
    check_encode_decode(dq8, kind, x, 0, tag="degenerate-pertensor")
    check_encode_decode(dq8, kind, x, 64, tag="degenerate-64")
    check_encode_decode(dq8, kind, x, 8192, tag="degenerate-8192")
    check_encode_decode(dq8, kind, x, 3 * 4096, tag="degenerate-12288")


@pytest.mark.parametrize("kind", KINDS)
def test_values_on_and_next_to_every_decision_point(dq8, kind):
    cb = np.unique(oracle.codebook(kind)[:128])  # ascending distinct magnitudes (the mantissa type repeats some)
    mid = ((cb[:-1].astype(np.float64) + cb[1:]) / 2).astype(np.float32).view(np.int32).astype(np.int64)
    near = (mid[:, None] + np.arange(-3, 4)[None, :]).reshape(-1).astype(np.int32).view(np.float32)
    pos = np.concatenate([near, cb, np.array([1.0], np.float32)])
    for scale in (1.0, 0.37, 3e-3, 1e20):
        x = np.concatenate([pos, -pos]) * np.float32(scale)
        x = np.concatenate([x, np.array([scale], np.float32)]).astype(np.float32)  # pins the absmax to `scale`
        check_encode_decode(dq8, kind, x, 0, tag="decision-points s=%g" % scale)


def test_all_codes_decode_and_reencode(dq8):
    for kind in KINDS:
        codes = np.arange(256, dtype=np.uint8)
        for s in (1.0, 3.0, 1e-3, 1e30):
            sc = np.array([s], np.float32)
            want = oracle.decode(kind, codes, sc, 0)
            got = dq8.decode(kind, dev(codes), dev(sc), 0)
            same_bits(got, want, "decode all codes")
            back, _ = dq8.encode(kind, dev(want), 0, scales=dev(sc), scales_given=True)
            canon, _ = oracle.encode(kind, want, 0, scales=sc)
            same_bits(back, canon, "encode(decode(c))")
            if kind != oracle.MANTISSA:  # every code is the only one of its value
                same_bits(back, codes, "encode(decode(c)) == c")
            else:  # the smallest code of the same sign and value
                cbk = oracle.codebook(kind)
                first = np.array([min(d for d in range(c & 0x80, (c & 0x80) + 128) if cbk[d] == cbk[c]) for c in range(256)])
                same_bits(back, first.astype(np.uint8), "encode(decode(c)) == smallest code of that value")


@pytest.mark.parametrize("kind", [2, 3])
def test_static_exponent_with_a_decade_offset(dq8, kind):
    """Sec. 3.1 shifts the static-exponent types by a fixed decade offset instead of normalising:
    that is the codec with the scale 10^offset handed in.  Values beyond the scale go to the
    nearest (largest) table value, which for the mantissa type lies above 1."""
    rng = np.random.Generator(np.random.PCG64(4100 + kind))
    n, block = 3 * 4096 + 500, 4096
    for offset in (-3, 0, 2):
        print("offset kind=%d 10^%d" % (kind, offset), flush=True)
        s = np.full(4, 10.0 ** offset, np.float32)
        x = (rng.standard_normal(n) * np.exp(rng.uniform(-12, 1, n)) * float(s[0])).astype(np.float32)
        want, _ = oracle.encode(kind, x, block, scales=s)
        got, _ = dq8.encode(kind, dev(x), block, scales=dev(s), scales_given=True)
        same_bits(got, want, "codes, decade offset %d" % offset)
        same_bits(dq8.decode(kind, got, dev(s), block), oracle.decode(kind, want, s, block), "decode, decade offset")


def check_error_stats(dq8, kind, x, block, given=None, tag=""):
    """Counts and maxima bit-exact; the sums are binary64 sums of non-negative terms in an order that is not
    fixed, so each side is within (terms) * 2^-53 (relative) of the real sum: tolerance 2 * terms * 2^-53."""
    print("error stats %s kind=%d n=%d block=%d given=%s" % (tag, kind, x.size, block, given is not None), flush=True)
    want, want_means = oracle.error_stats(kind, x, block, scales=given)
    nb = want.shape[0]
    gs = Guarded(nb, np.float32, data=given)
    gstats = torch.full((nb + 2, 4), 7.0, dtype=torch.float64, device="cuda")
    gmeans = torch.full((6,), 7.0, dtype=torch.float64, device="cuda")
    stats, means = dq8.error_stats(kind, dev(x), block, scales=gs.t, scales_given=given is not None,
                                   stats=gstats[1:nb + 1], means=gmeans[2:4])
    gs.check("error stats scales")
    got, got_means = stats.cpu().numpy(), means.cpu().numpy()
    assert bool((gstats[0] == 7.0).all()) and bool((gstats[nb + 1] == 7.0).all()), "stats margins written"
    assert bool((gmeans[:2] == 7.0).all()) and bool((gmeans[4:] == 7.0).all()), "means margins written"
    if given is None:
        same_bits(gs.t, oracle.absmax(x, block), "error stats scales " + tag)
    B = x.size if block == 0 or block > x.size else block
    terms = np.minimum(B, x.size - B * np.arange(nb)).astype(np.float64)
    assert got[:, 2].tobytes() == want[:, 2].tobytes(), "non-zero counts " + tag
    assert got[:, 3].tobytes() == want[:, 3].tobytes(), "largest errors " + tag
    for col in (0, 1):
        tol = 2 * terms * 2.0 ** -53 * want[:, col]
        bad = np.nonzero(np.abs(got[:, col] - want[:, col]) > tol)[0]
        assert bad.size == 0, (tag, col, bad[:5], got[bad[:5], col], want[bad[:5], col])
    tol = 4 * x.size * 2.0 ** -53
    assert np.all(np.abs(got_means - want_means) <= tol * want_means), (tag, got_means, want_means)
    return got


@pytest.mark.parametrize("kind", KINDS)
def test_error_stats_per_element_are_bit_exact(dq8, kind):
    """Blocks of one element: every sum has a single term, so all four columns are exact."""
    rng = np.random.Generator(np.random.PCG64(5100 + kind))
    n = 5000
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-10, 3, n))).astype(np.float32)
    x[::13] = 0.0
    x[5::29] = -0.0
    given = np.full(n, 16.0, np.float32)
    want, _ = oracle.error_stats(kind, x, 1, scales=given)
    stats, _ = dq8.error_stats(kind, dev(x), 1, scales=dev(given), scales_given=True)
    same_bits(stats.reshape(-1), want.reshape(-1), "per-element error statistics")
    want, _ = oracle.error_stats(kind, x, 1)  # own absmax: every element is its own scale
    stats, _ = dq8.error_stats(kind, dev(x), 1)
    same_bits(stats.reshape(-1), want.reshape(-1), "per-element error statistics, own scale")


@pytest.mark.parametrize("kind", KINDS)
def test_error_stats_shapes(dq8, kind):
    for i, (n, block) in enumerate(SHAPES):
        x = workloads.edge_case_block("wide", n, seed=7000 + 10 * kind + i)
        x[::11] = 0.0
        check_error_stats(dq8, kind, x, block, tag="shape%d" % i)
    n = 3 * 4096 + 77
    x = workloads.edge_case_block("wide", n, seed=7100 + kind)
    for off in (1, 3):  # misaligned input
        want, _ = oracle.error_stats(kind, x, 4096)
        got, _ = dq8.error_stats(kind, dev(x, off), 4096)
        got = got.cpu().numpy()
        assert got[:, 2:].tobytes() == want[:, 2:].tobytes()
        assert np.allclose(got[:, :2], want[:, :2], rtol=1e-12, atol=0)
    z = np.zeros(5000, np.float32)
    z[100:200] = -0.0
    got = check_error_stats(dq8, kind, z, 1024, tag="zeros")
    assert np.all(got == 0)


@pytest.mark.parametrize("kind", KINDS)
def test_error_stats_when_wavefronts_own_whole_blocks(dq8, kind):
    """With at least one block per resident wavefront (6144 on this GPU) and blocks of at most 64 units, a wavefront
    owns whole blocks: plain stores into rows that were never zeroed, a fixed order of summation.  Blocks of one
    element (every column exact), blocks shorter than a unit, of one unit, of three units with a short last one, of
    four units; a ragged last block; a misaligned input; and the same bits from two launches."""
    rng = np.random.Generator(np.random.PCG64(5300 + kind))
    n = 7001
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-10, 3, n))).astype(np.float32)
    x[::13] = 0.0
    want, _ = oracle.error_stats(kind, x, 1)
    stats, _ = dq8.error_stats(kind, dev(x), 1)
    same_bits(stats.reshape(-1), want.reshape(-1), "per-element error statistics, owned blocks")
    for i, (nb, block, tail) in enumerate([(6200, 100, 37), (6150, 1024, 500), (6145, 3000, 8), (6144, 4096, 808)]):
        n = nb * block + tail
        x = (rng.standard_normal(n) * np.exp(rng.uniform(-6, 0, n))).astype(np.float32)
        x[::17] = 0.0
        check_error_stats(dq8, kind, x, block, tag="owned%d" % i)
        if i == 3 and kind == 0:
            a, ma = dq8.error_stats(kind, dev(x), block)
            b, mb = dq8.error_stats(kind, dev(x), block)
            assert torch.equal(a, b) and torch.equal(ma, mb), "owned blocks are summed in a fixed order"
            want, _ = oracle.error_stats(kind, x, block)
            got, _ = dq8.error_stats(kind, dev(x, 1), block)  # input one element off a 16-byte boundary
            got = got.cpu().numpy()
            assert got[:, 2:].tobytes() == want[:, 2:].tobytes()
            assert np.allclose(got[:, :2], want[:, :2], rtol=1e-12, atol=0)


def test_error_stats_of_the_table_2_samples(dq8):
    """Sec. 3.4: samples from U(0,1) and normal distributions; static-exponent types with a decade as scale."""
    rng = np.random.Generator(np.random.PCG64(5200))
    n = 300000
    data = {"U(0,1)": (rng.random(n), 1), "N(0,1)": (rng.standard_normal(n), 1),
            "N(0,10^2)": (10 * rng.standard_normal(n), 2), "N(0,0.2^2)": (0.2 * rng.standard_normal(n), 1)}
    for name, (xs, offset) in data.items():
        x = xs.astype(np.float32)
        for kind in (oracle.DYNAMIC_TREE, oracle.LINEAR):
            check_error_stats(dq8, kind, x, 0, tag=name)
        for kind in (oracle.STATIC_TREE, oracle.MANTISSA):
            check_error_stats(dq8, kind, x, 0, given=np.array([10.0 ** offset], np.float32), tag=name)
            check_error_stats(dq8, kind, x, 4096, given=np.full((n + 4095) // 4096, 10.0 ** offset, np.float32), tag=name)


AVG_CASES = [(2 * 4096 + 333, 4096, 0), (3 * 4096, 4096, 0), (10000, 0, 0), (3000, 1000, 0), (4096 * 3, 4096, 1),
             (100, 7, 0), (4096, 0, 0), (4095, 0, 0),
             (5 * 1024 + 100, 1024, 0),   # two whole units per block, ragged last unit
             (3 * 1536, 1536, 0),         # three units per block: not a power of two
             (3 * 2048 + 7, 2048, 0), (40 * 512, 512, 0), (511, 0, 0), (512, 0, 0), (513, 0, 0),
             (20 * 256 + 12, 256, 0), (64 * 64, 64, 0), (7 * 1000 + 4, 1000, 0), (5 * 516 + 2, 516, 0),
             (3 * 1000, 1000, 2),     # short blocks: aligned (whole quads), with a tail, and misaligned
             (5 * 1024 + 300, 64, 0), (3 * 1024 + 12, 4, 0), (4 * 1024, 128, 0), (2 * 1024 + 64, 32, 1),
             (6 * 1024 + 8, 8, 0), (2 * 1024 + 16, 16, 0),  # blocks of 4 .. 128 elements
             # blocks of whole quads that are not a power-of-two number of units: units by position, two scales each
             (40 * 1000 + 300, 1000, 0), (9 * 3000 + 8, 3000, 0), (5 * 9216 + 100, 9216, 0), (24 * 516, 516, 0)]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6, 7, 8, 32])
def test_decode_accumulate_avg(dq8, kind, K):
    rng = np.random.Generator(np.random.PCG64(900 + 10 * K + kind))
    for n, block, off in AVG_CASES:
        print("avg kind=%d K=%d n=%d block=%d off=%d" % (kind, K, n, block, off), flush=True)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
        sl = [np.exp(rng.uniform(-8, 8, nb)).astype(np.float32) for _ in range(K)]
        want = oracle.decode_accumulate_avg(kind, cl, sl, block)
        go = Guarded(n, np.float32, off)
        got = dq8.decode_accumulate_avg(kind, [dev(c, off) for c in cl], [dev(s) for s in sl], block, out=go.t)
        same_bits(got, want, "avg")
        go.check("avg")




@pytest.mark.parametrize("K", range(9, 33))
def test_decode_accumulate_avg_many_workers(dq8, K):
    """Every worker count above 8: the workers are taken a chunk at a time over the same sums, the last chunk
    with empty places; several units per wavefront and a ragged tail."""
    kind = KINDS[K % len(KINDS)]
    rng = np.random.Generator(np.random.PCG64(5900 + K))
    for n, block in [(40 * 4096 + 333, 4096), (9 * 1024 + 5, 1024), (3 * 512, 0), (2100 * 512 + 12, 2048),
                     (30 * 1000 + 100, 1000), (7 * 3000, 3000), (20 * 256 + 4, 256)]:  # and units by position
        print("avg many kind=%d K=%d n=%d block=%d" % (kind, K, n, block), flush=True)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
        sl = [np.exp(rng.uniform(-8, 8, nb)).astype(np.float32) for _ in range(K)]
        want = oracle.decode_accumulate_avg(kind, cl, sl, block)
        go = Guarded(n, np.float32, 0)
        got = dq8.decode_accumulate_avg(kind, [dev(c) for c in cl], [dev(s) for s in sl], block, out=go.t)
        same_bits(got, want, "avg many")
        go.check("avg many")


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("K", [0, 1, 2, 3, 4, 5, 6, 7, 8, 32])
def test_decode_accumulate_avg_with_local_term(dq8, kind, K):
    """The caller's own fp32 gradient is the first of K + 1 terms."""
    rng = np.random.Generator(np.random.PCG64(1900 + 10 * K + kind))
    for n, block, off in AVG_CASES:
        print("avg+local kind=%d K=%d n=%d block=%d off=%d" % (kind, K, n, block, off), flush=True)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
        sl = [np.exp(rng.uniform(-8, 8, nb)).astype(np.float32) for _ in range(K)]
        local = (rng.standard_normal(n) * np.exp(rng.uniform(-8, 8, n))).astype(np.float32)
        local[::17] = 0.0
        local[5::23] = -0.0
        want = oracle.decode_accumulate_avg(kind, cl, sl, block, local=local)
        go = Guarded(n, np.float32, off)
        got = dq8.decode_accumulate_avg(kind, [dev(c, off) for c in cl], [dev(s) for s in sl], block, out=go.t,
                                        local=dev(local, off))
        same_bits(got, want, "avg+local")
        go.check("avg+local")


# every type with up to 8 workers and with 32; the worker counts that take several passes with two types
FUSED_CASES = [(kind, K, wl) for kind in KINDS for K, wl in [(1, False), (2, False), (3, False), (8, False), (32, False),
                                                             (0, True), (3, True), (7, True)]] + \
              [(kind, K, wl) for kind in (0, 3) for K, wl in [(9, False), (12, True), (13, False), (16, False), (31, True)]]


@pytest.mark.parametrize("kind,K,with_local", FUSED_CASES)
def test_decode_avg_encode(dq8, kind, K, with_local):
    """One call: average, then compress the average.  Inputs are codes of seeded gradients (so that the means
    spread over the whole table) and, for the ragged shapes, random codes."""
    rng = np.random.Generator(np.random.PCG64(2900 + 10 * K + kind + 1000 * with_local))
    for n, block, off in AVG_CASES:
        Bq = n if block == 0 else block
        if Bq > 4096:
            continue
        print("avg->encode kind=%d K=%d local=%d n=%d block=%d off=%d" % (kind, K, with_local, n, block, off), flush=True)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        if n >= 4096:
            enc = [oracle.encode(kind, workloads.tensor(5, 2, worker=w, limit=n), block) for w in range(K)]
            cl, sl = [e[0] for e in enc], [e[1] for e in enc]
        else:
            cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
            sl = [np.exp(rng.uniform(-8, 8, nb)).astype(np.float32) for _ in range(K)]
        local = (workloads.tensor(5, 4, worker=9, limit=n) if n >= 4096 else rng.standard_normal(n).astype(np.float32)) \
            if with_local else None
        if n == 3 * 4096:  # one block whose average is zero everywhere, one with a denormal maximum
            if K >= 2 and not with_local:
                cl[1][:4096] = cl[0][:4096] ^ np.uint8(0x80)
                sl[1][0] = sl[0][0]
                for k in range(2, K):  # the other workers contribute +-0 to that block
                    sl[k][0] = 0.0
            for k in range(K):
                sl[k][1] = np.float32(1e-42)
                sl[k][2] = np.float32(2.0 ** 110) if k % 2 else np.float32(2.0 ** 101)  # sums far above the usual range
            if with_local:
                local[4096:8192] = np.float32(3e-43)
        want_codes, want_scales = oracle.decode_avg_encode(kind, cl, sl, block, local=local)
        gc, gs = Guarded(n, np.uint8, off), Guarded(nb, np.float32)
        codes, scales = dq8.decode_avg_encode(kind, [dev(c, off) for c in cl], [dev(s) for s in sl], block,
                                              local=None if local is None else dev(local, off), scales=gs.t, codes=gc.t)
        same_bits(scales, want_scales, "avg->encode scales")
        same_bits(codes, want_codes, "avg->encode codes")
        gc.check("avg->encode codes")
        gs.check("avg->encode scales")


@pytest.mark.parametrize("seed", range(int(os.environ.get("DQ8_RANDOM_SEEDS", "6"))))
def test_random_shapes_through_every_call(dq8, seed):
    """Seeded random sizes, block lengths, pointer offsets, worker counts and data types through every call:
    the launch logic picks unit sizes and kernel variants from these, so this sweeps their combinations."""
    rng = np.random.Generator(np.random.PCG64(8800 + seed))
    for case in range(10):
        n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 6000), rng.integers(6000, 40000)]))
        if case == 0:  # one size per seed at which every wavefront walks several units
            n = int(rng.integers(1_500_000, 3_000_000))
        pick = rng.integers(0, 7)
        block = [0, int(rng.integers(1, n + 1)), 4 * int(rng.integers(1, max(2, n // 4 + 1))),
                 1 << int(rng.integers(0, 15)), 4096, int(rng.integers(1, 9)) * 1000,
                 4 * int(rng.integers(1025, 4097))][pick]  # the last: blocks that a team holds in 6 to 16 quads per lane
        kind = int(rng.integers(0, 4))
        x_off, c_off = int(rng.integers(0, 4)) * int(rng.integers(0, 2)), int(rng.integers(0, 4)) * int(rng.integers(0, 2))
        K = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 17]))
        with_local = bool(rng.integers(0, 2))
        tag = "random seed=%d case=%d n=%d block=%d kind=%d x_off=%d c_off=%d K=%d local=%d" % (
            seed, case, n, block, kind, x_off, c_off, K, with_local)
        x = (rng.standard_normal(n) * np.exp(rng.uniform(-9, 2, n))).astype(np.float32)
        x[rng.random(n) < 0.05] = 0.0
        check_encode_decode(dq8, kind, x, block, x_off=x_off, c_off=c_off, tag=tag)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
        sl = [np.exp(rng.uniform(-8, 8, nb)).astype(np.float32) for _ in range(K)]
        local = (rng.standard_normal(n) * np.exp(rng.uniform(-8, 8, n))).astype(np.float32) if with_local else None
        want = oracle.decode_accumulate_avg(kind, cl, sl, block, local=local)
        go = Guarded(n, np.float32, x_off)
        got = dq8.decode_accumulate_avg(kind, [dev(c, c_off) for c in cl], [dev(s_) for s_ in sl], block, out=go.t,
                                        local=None if local is None else dev(local, x_off))
        same_bits(got, want, "avg " + tag)
        go.check("avg " + tag)
        if (n if block == 0 or block > n else block) <= 16384:
            want_codes, want_scales = oracle.decode_avg_encode(kind, cl, sl, block, local=local)
            gc, gs = Guarded(n, np.uint8, c_off), Guarded(nb, np.float32)
            codes, scales = dq8.decode_avg_encode(kind, [dev(c, c_off) for c in cl], [dev(s_) for s_ in sl], block,
                                                  local=None if local is None else dev(local, x_off), scales=gs.t,
                                                  codes=gc.t)
            same_bits(scales, want_scales, "avg->encode scales " + tag)
            same_bits(codes, want_codes, "avg->encode codes " + tag)
            gc.check("avg->encode " + tag)
            gs.check("avg->encode " + tag)
        check_error_stats(dq8, kind, x, block, tag=tag)
        # the same array cut at random places, one scale per piece
        n_seg = int(rng.integers(1, 40))
        cuts = np.sort(rng.integers(0, n + 1, n_seg - 1))
        check_segments(dq8, kind, x, np.concatenate([[0], cuts, [n]]), x_off=x_off, c_off=c_off, tag=tag)


def test_decode_avg_encode_rejects_blocks_that_do_not_fit(dq8):
    c = torch.zeros(20000, dtype=torch.uint8, device="cuda")
    s = torch.ones(1, device="cuda")
    with pytest.raises(dq8.Dq8Error, match="16384"):
        dq8.decode_avg_encode(0, [c, c], [s, s], 0)


LONG_FUSED_SHAPES = [(3 * 8192 + 100, 8192, 0), (2 * 16384 + 5000, 16384, 0), (3 * 9216 + 4, 9216, 0), (10000, 0, 0),
                     (2 * 4100, 4100, 0), (2 * 8191 + 3, 8191, 0),  # blocks that are not whole quads
                     (2 * 12288 + 40, 12288, 1), (5000, 0, 3)]      # misaligned buffers


@pytest.mark.parametrize("kind,K,with_local", [(0, 1, False), (0, 2, False), (1, 3, True), (2, 8, False), (3, 7, True),
                                               (0, 0, True), (3, 13, False), (0, 32, True)])
def test_decode_avg_encode_long_blocks(dq8, kind, K, with_local):
    """Blocks of 4097 .. 16384 elements: a workgroup per block."""
    rng = np.random.Generator(np.random.PCG64(7900 + 10 * K + kind))
    for n, block, off in LONG_FUSED_SHAPES:
        print("avg->encode long kind=%d K=%d local=%d n=%d block=%d off=%d" % (kind, K, with_local, n, block, off), flush=True)
        nb = oracle.dq8_oracle.n_blocks(n, block)
        enc = [oracle.encode(kind, workloads.tensor(5, 2, worker=w, limit=n), block) for w in range(K)]
        cl, sl = [e[0] for e in enc], [e[1] for e in enc]
        local = workloads.tensor(5, 4, worker=9, limit=n) if with_local else None
        if K >= 2 and not with_local:  # the first block's average is zero everywhere
            B = n if block == 0 else block
            cl[1][:B] = cl[0][:B] ^ np.uint8(0x80)
            sl[1][0] = sl[0][0]
            for k in range(2, K):
                sl[k][0] = 0.0
        want_codes, want_scales = oracle.decode_avg_encode(kind, cl, sl, block, local=local)
        gc, gs = Guarded(n, np.uint8, off), Guarded(nb, np.float32)
        codes, scales = dq8.decode_avg_encode(kind, [dev(c, off) for c in cl], [dev(s) for s in sl], block,
                                              local=None if local is None else dev(local, off), scales=gs.t, codes=gc.t)
        same_bits(scales, want_scales, "avg->encode long scales")
        same_bits(codes, want_codes, "avg->encode long codes")
        gc.check("avg->encode long codes")
        gs.check("avg->encode long scales")


@pytest.mark.parametrize("kind,K,with_local,n,block", [
    (0, 8, False, 1300 * 4100 + 52, 4100),   # a short last block of whole quads
    (3, 5, True, 700 * 8192 + 8191, 8192),   # a last block that is not whole quads
    (1, 13, False, 600 * 5000, 5000),        # more workers than register sets, a third of the lanes' last quads unused
    (2, 3, False, 520 * 16384 + 12, 16384),  # fewer workers than register sets
    (0, 1, True, 1100 * 6148, 6148),
    (0, 7, True, 520 * 12288 + 8, 12288),    # one register set short of the workers, four sets rotate
    (1, 4, False, 900 * 9216, 9216),
    (2, 2, True, 530 * 7000, 7000),
    (3, 7, False, 1400 * 4104 + 400, 4104),
    # blocks of 513 .. 3072 elements: teams of one, two or three wavefronts, more blocks than teams
    (0, 8, False, 7000 * 1024 + 500, 1024), (3, 8, False, 3300 * 2048, 2048), (1, 8, True, 2500 * 3000 + 8, 3000),
    (2, 8, False, 7100 * 1000 + 3, 1000), (0, 8, False, 2300 * 3072 + 1, 3072), (0, 8, False, 4000 * 1600, 1600),
    (1, 4, False, 3200 * 2048 + 100, 2048), (2, 2, True, 7000 * 1000, 1000), (3, 3, False, 2400 * 3000 + 4, 3000),
    (0, 7, True, 6500 * 1024, 1024), (0, 1, False, 7000 * 1024, 1024), (3, 5, True, 3300 * 2000, 2000),
    (1, 6, False, 2400 * 3072, 3072), (2, 6, False, 600 * 10000, 10000)])
def test_decode_avg_encode_several_blocks_per_team(dq8, kind, K, with_local, n, block):
    """More blocks than workgroups (long blocks) or teams of wavefronts (shorter ones): each walks several blocks and
    requests the next block's code words while it finishes the current one."""
    print("avg->encode, many blocks kind=%d K=%d local=%d n=%d block=%d" % (kind, K, with_local, n, block), flush=True)
    nb = oracle.dq8_oracle.n_blocks(n, block)
    enc = [oracle.encode(kind, workloads.tensor(5, 12, worker=w, limit=n), block) for w in range(K)]
    cl, sl = [e[0] for e in enc], [e[1] for e in enc]
    local = workloads.tensor(5, 12, worker=9, limit=n) if with_local else None
    want_codes, want_scales = oracle.decode_avg_encode(kind, cl, sl, block, local=local)
    gc, gs = Guarded(n, np.uint8), Guarded(nb, np.float32)
    codes, scales = dq8.decode_avg_encode(kind, [dev(c) for c in cl], [dev(s) for s in sl], block,
                                          local=None if local is None else dev(local), scales=gs.t, codes=gc.t)
    same_bits(scales, want_scales, "avg->encode long scales")
    same_bits(codes, want_codes, "avg->encode long codes")
    gc.check("avg->encode long codes")
    gs.check("avg->encode long scales")


def test_average_order_is_worker_zero_first(dq8):
    c_pos, c_neg = np.full(5000, 127, np.uint8), np.full(5000, 255, np.uint8)
    big, small = np.array([1e8], np.float32), np.array([1.0], np.float32)
    for cl, sl in [([c_pos, c_neg, c_pos], [big, big, small]), ([c_pos, c_pos, c_neg], [big, small, big])]:
        want = oracle.decode_accumulate_avg(oracle.LINEAR, cl, sl, 0)
        got = dq8.decode_accumulate_avg(oracle.LINEAR, [dev(c) for c in cl], [dev(s) for s in sl], 0)
        same_bits(got, want, "order")


def test_config1_mnist_mlp_gradients(dq8):
    for name, x in workloads.tensors(1):
        check_encode_decode(dq8, 0, x, 0, tag="C1 " + name)


def test_config2_convnet_gradients_all_types(dq8):
    for kind in KINDS:
        for name, x in workloads.tensors(2):
            check_encode_decode(dq8, kind, x, 0, tag="C2 %s %s" % (NAMES[kind], name))


def test_config4_activations_per_row(dq8):
    for name, x in workloads.tensors(4):
        check_encode_decode(dq8, 0, x, 4096, tag="C4 " + name)
        # a rectified row of zeros encodes to code 0 and decodes to +0
        assert np.mean(x == 0) > 0.45


def test_errors_are_reported(dq8):
    x = torch.zeros(100, device="cuda")
    with pytest.raises(dq8.Dq8Error):
        dq8.encode(7, x)
    codes = torch.zeros(400, dtype=torch.uint8, device="cuda")
    with pytest.raises(dq8.Dq8Error):  # out overlapping an input
        dq8.lib().dq8_last_error()
        rc = dq8.lib().dq8_decode(0, x.data_ptr(), x.data_ptr(), 100, 0, x.data_ptr(), None)
        dq8._check(rc, "dq8_decode")
    del codes


def test_a_captured_graph_of_the_whole_path_replays_exactly(dq8):
    """The calls launch kernels only (no allocation, no memset, no synchronisation once the tables are on the
    device), so a caller can capture them in a HIP graph.  A graph of the whole path is replayed several times
    on new inputs, with eager work and synchronisations in between, and every replay must equal the oracle."""
    kind, B, K = oracle.DYNAMIC_TREE, 4096, 4
    n = 6 * B + 1000
    nb = oracle.dq8_oracle.n_blocks(n, B)
    x = torch.zeros(n, device="cuda")
    codes_in = [torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(K)]
    scales_in = [torch.ones(nb, device="cuda") for _ in range(K)]
    amax = torch.empty(nb, device="cuda")
    codes, scales = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(nb, device="cuda")
    dec, mean = torch.empty(n, device="cuda"), torch.empty(n, device="cuda")
    rcodes, rscales = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(nb, device="cuda")
    fcodes, fscales = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(nb, device="cuda")
    whole = torch.empty(1, device="cuda")
    stats, means = torch.empty((nb, 4), dtype=torch.float64, device="cuda"), torch.empty(2, dtype=torch.float64, device="cuda")
    sscales = torch.empty(nb, device="cuda")

    def path():
        dq8.absmax(x, B, scales=amax)
        dq8.absmax(x, 0, scales=whole)  # several units per block: zero fill + atomics
        dq8.encode(kind, x, B, scales=scales, codes=codes)
        dq8.decode(kind, codes, scales, B, out=dec)
        dq8.decode_accumulate_avg(kind, codes_in, scales_in, B, out=mean)
        dq8.encode(kind, mean, B, scales=rscales, codes=rcodes)
        dq8.decode_avg_encode(kind, codes_in, scales_in, B, scales=fscales, codes=fcodes)
        dq8.error_stats(kind, x, B, scales=sscales, stats=stats, means=means)

    path()  # warm-up outside the capture: tables are uploaded on first use
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        path()
    for rep in range(3):
        xs = workloads.tensor(5, 2, worker=rep, limit=n)
        enc = [oracle.encode(kind, workloads.tensor(5, 2, worker=10 * (rep + 1) + k, limit=n), B) for k in range(K)]
        x.copy_(torch.from_numpy(xs))
        for k in range(K):
            codes_in[k].copy_(torch.from_numpy(enc[k][0]))
            scales_in[k].copy_(torch.from_numpy(enc[k][1]))
        for t in (amax, codes, scales, dec, mean, rcodes, rscales, fcodes, fscales, whole, sscales):
            t.zero_()  # eager work between replays; stale results would show
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        print("graph replay %d" % rep, flush=True)
        wc, ws = oracle.encode(kind, xs, B)
        same_bits(amax, ws, "graph absmax")
        same_bits(whole, oracle.absmax(xs, 0), "graph absmax of the whole array")
        same_bits(codes, wc, "graph codes")
        same_bits(scales, ws, "graph scales")
        same_bits(dec, oracle.decode(kind, wc, ws, B), "graph decode")
        wm = oracle.decode_accumulate_avg(kind, [e[0] for e in enc], [e[1] for e in enc], B)
        same_bits(mean, wm, "graph mean")
        wrc, wrs = oracle.encode(kind, wm, B)
        same_bits(rcodes, wrc, "graph re-encoded codes")
        same_bits(rscales, wrs, "graph re-encoded scales")
        same_bits(fcodes, wrc, "graph one-call codes")
        same_bits(fscales, wrs, "graph one-call scales")
        wst, wmeans = oracle.error_stats(kind, xs, B)
        got = stats.cpu().numpy()
        assert got[:, 2:].tobytes() == wst[:, 2:].tobytes()
        assert np.allclose(got[:, :2], wst[:, :2], rtol=1e-12, atol=0)
        assert np.allclose(means.cpu().numpy(), wmeans, rtol=1e-12, atol=0)


def test_table_2_script_rows(dq8):
    """The script that reproduces the synthetic rows of Table 2 (Sec. 3.4): 16 rows, the dynamic tree has the
    smallest relative error on every distribution (the paper's bold entries), ratios to the printed values
    in the same band as the oracle's."""
    from paper_1511_04561_amd import table2
    rows = table2.rows(samples=400000, seed=7)
    assert len(rows) == 16
    by_dist = {}
    for name, label, mae, mre, worst in rows:
        by_dist.setdefault(name, {})[label] = mre
        assert mae > 0 and worst >= mae
    for name, d in by_dist.items():
        assert min(d, key=d.get) == "8-bit dynamic tree", (name, d)
    printed = {}
    for l in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table2_mre_all_types.txt")):
        if l.strip() and l[0] != "#":
            dist, typ, v, _ = l.split()
            printed[(dist, typ)] = float(v)
    names = {"8-bit dynamic tree": "dynamic_tree", "8-bit linear quant": "linear", "8-bit mantissa": "mantissa",
             "8-bit static tree": "static_tree"}
    for name, label, mae, mre, worst in rows:
        assert 0.6 < mre / printed[(name, names[label])] < 0.9, (name, label, mre)


@pytest.mark.parametrize("kind", KINDS)
def test_non_finite_inputs_stay_inside_their_block(dq8, kind):
    """Inputs are required to be finite.  NaN and infinities must still leave every call in bounds (the code
    search clamps its key) and must not disturb other blocks: those still equal the oracle."""
    B = 4096
    n = 5 * B + 100
    x = workloads.edge_case_block("wide", n, seed=300 + kind)
    bad = x.copy()
    bad[B + 5] = np.nan
    bad[B + 900] = -np.inf
    bad[3 * B + 1] = np.inf
    codes, scales = dq8.encode(kind, dev(bad), B)
    amax = dq8.absmax(dev(bad), B)
    out = dq8.decode(kind, codes, scales, B)
    mean = dq8.decode_accumulate_avg(kind, [codes, codes], [scales, scales], B)
    fc, fs = dq8.decode_avg_encode(kind, [codes, codes], [scales, scales], B)
    stats, _ = dq8.error_stats(kind, dev(bad), B)
    torch.cuda.synchronize()
    wc, ws = oracle.encode(kind, x, B)
    wo = oracle.decode(kind, wc, ws, B)
    wm = oracle.decode_accumulate_avg(kind, [wc, wc], [ws, ws], B)
    wfc, wfs = oracle.encode(kind, wm, B)
    wst, _ = oracle.error_stats(kind, x, B)
    for b in (0, 2, 4, 5):  # the blocks without a non-finite value
        lo, hi = b * B, min(n, (b + 1) * B)
        same_bits(codes[lo:hi], wc[lo:hi], "codes of a clean block")
        same_bits(scales[b:b + 1], ws[b:b + 1], "scale of a clean block")
        same_bits(amax[b:b + 1], ws[b:b + 1], "absmax of a clean block")
        same_bits(out[lo:hi], wo[lo:hi], "decode of a clean block")
        same_bits(mean[lo:hi], wm[lo:hi], "mean of a clean block")
        same_bits(fc[lo:hi], wfc[lo:hi], "compressed mean of a clean block")
        same_bits(fs[b:b + 1], wfs[b:b + 1], "scale of the compressed mean of a clean block")
        got = stats[b].cpu().numpy()
        assert got[2:].tobytes() == wst[b, 2:].tobytes() and np.allclose(got[:2], wst[b, :2], rtol=1e-12, atol=0)


def test_calls_from_several_threads_on_their_own_streams(dq8):
    """The library keeps no per-call state outside the caller's buffers: threads that launch on their own
    streams at the same time (ctypes releases the interpreter lock during a call) get the same bits as the
    oracle."""
    import threading
    kind, B, n, rounds = oracle.DYNAMIC_TREE, 4096, 9 * 4096 + 123, 12
    xs = [workloads.tensor(5, 2, worker=40 + t, limit=n) for t in range(4)]
    want = [oracle.encode(kind, x, B) for x in xs]
    want_dec = [oracle.decode(kind, c, s, B) for c, s in want]
    errors = []

    def work(t):
        try:
            stream = torch.cuda.Stream()
            xd = torch.from_numpy(xs[t]).cuda()
            with torch.cuda.stream(stream):
                for r in range(rounds):
                    codes, scales = dq8.encode(kind, xd, B)
                    out = dq8.decode(kind, codes, scales, B)
                    mean = dq8.decode_accumulate_avg(kind, [codes, codes], [scales, scales], B)
                    stream.synchronize()
                    if codes.cpu().numpy().tobytes() != want[t][0].tobytes() or \
                            scales.cpu().numpy().tobytes() != want[t][1].tobytes() or \
                            out.cpu().numpy().tobytes() != want_dec[t].tobytes() or \
                            mean.cpu().numpy().tobytes() != (want_dec[t] + np.float32(0)).tobytes():
                        errors.append("thread %d round %d differs from the oracle" % (t, r))
                        return
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append("thread %d: %r" % (t, e))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a thread did not finish"
    assert errors == []


def test_debug_switch_waits_after_every_launch(dq8):
    """DQ8_DEBUG=1 is read once per process, so the round trip runs in a process of its own: every call waits for
    its kernels and checks the device's error state; results are the oracle's bits, and the work of a call is
    finished when the call returns (the outputs are read without any synchronisation in between)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    script = r"""
import sys
sys.path.insert(0, %r)
import numpy as np, torch, oracle
from paper_1511_04561_amd import dq8, workloads
n, B = 40 * 4096 + 77, 4096
x = workloads.tensor(5, 2, worker=3, limit=n)
stream = torch.cuda.Stream()
with torch.cuda.stream(stream):
    xd = torch.from_numpy(x).cuda()
    stream.synchronize()
    for kind in (0, 3):
        codes, scales = dq8.encode(kind, xd, B)
        done = stream.query()          # nothing may be pending on the stream once the call has returned
        out = dq8.decode(kind, codes, scales, B)
        done = done and stream.query()
        mean = dq8.decode_accumulate_avg(kind, [codes, codes, codes], [scales, scales, scales], B)
        done = done and stream.query()
        fc, fs = dq8.decode_avg_encode(kind, [codes, codes, codes], [scales, scales, scales], B)
        done = done and stream.query()
        stats, means = dq8.error_stats(kind, xd, B)
        done = done and stream.query()
        assert done, "a call returned before its kernels had finished"
        wc, ws = oracle.encode(kind, x, B)
        assert codes.cpu().numpy().tobytes() == wc.tobytes() and scales.cpu().numpy().tobytes() == ws.tobytes()
        assert out.cpu().numpy().tobytes() == oracle.decode(kind, wc, ws, B).tobytes()
        wm = oracle.decode_accumulate_avg(kind, [wc] * 3, [ws] * 3, B)
        assert mean.cpu().numpy().tobytes() == wm.tobytes()
        oc, os_ = oracle.encode(kind, wm, B)
        assert fc.cpu().numpy().tobytes() == oc.tobytes() and fs.cpu().numpy().tobytes() == os_.tobytes()
        assert stats.cpu().numpy()[:, 2].tobytes() == oracle.error_stats(kind, x, B)[0][:, 2].tobytes()
print("debug round trip ok")
""" % root
    env = dict(os.environ, DQ8_DEBUG="1")
    p = subprocess.run([sys.executable, "-c", script], env=env, capture_output=True, text=True, timeout=600)
    assert p.returncode == 0 and "debug round trip ok" in p.stdout, p.stdout[-2000:] + p.stderr[-4000:]


# ---- tensors back to back in one array, one scale per tensor

def bounds_dev(b):
    return torch.from_numpy(np.asarray(b, dtype=np.int64)).cuda()


def check_segments(dq8, kind, x, bounds, x_off=0, c_off=0, tag=""):
    """absmax, encode (scales computed and handed in) and decode of a segmented array against the oracle's
    per-segment results, with guard bands around every output."""
    n, n_seg = x.size, len(bounds) - 1
    print("segments %s kind=%d n=%d segments=%d x_off=%d c_off=%d" % (tag, kind, n, n_seg, x_off, c_off), flush=True)
    want_codes, want_scales = oracle.encode_segments(kind, x, bounds)
    want_out = oracle.decode_segments(kind, want_codes, want_scales, bounds)
    b = bounds_dev(bounds)
    xd = dev(x, x_off)
    gs = Guarded(n_seg, np.float32)
    dq8.absmax_segments(xd, b, scales=gs.t)
    same_bits(gs.t, want_scales, "segment maxima " + tag)
    gs.check("segment maxima " + tag)
    gc, gs2 = Guarded(n, np.uint8, c_off), Guarded(n_seg, np.float32)
    dq8.encode_segments(kind, xd, b, scales=gs2.t, codes=gc.t)
    same_bits(gs2.t, want_scales, "segment scales " + tag)
    same_bits(gc.t, want_codes, "segment codes " + tag)
    gc.check("segment codes " + tag)
    gs2.check("segment scales " + tag)
    # scales handed in: twice the maxima (a power of two: the quotients halve exactly)
    given = (2.0 * want_scales).astype(np.float32)
    want_c2, _ = oracle.encode_segments(kind, x, bounds, scales=given)
    gc2 = Guarded(n, np.uint8, c_off)
    dq8.encode_segments(kind, xd, b, scales=dev(given), codes=gc2.t, scales_given=True)
    same_bits(gc2.t, want_c2, "segment codes, scales given " + tag)
    gc2.check("segment codes, scales given " + tag)
    go = Guarded(n, np.float32, x_off)
    dq8.decode_segments(kind, dev(want_codes, c_off), dev(want_scales), b, out=go.t)
    same_bits(go.t, want_out, "segment decode " + tag)
    go.check("segment decode " + tag)


@pytest.mark.parametrize("kind", KINDS)
def test_segments_of_the_gradient_sets(dq8, kind):
    """The MLP's and the small convnet's gradient tensors back to back: one call for the whole set, results equal
    to one call per tensor."""
    for config in (1, 2):
        parts = [t for _, t in workloads.tensors(config)]
        bounds = np.concatenate([[0], np.cumsum([p.size for p in parts])])
        check_segments(dq8, kind, np.concatenate(parts), bounds, tag="C%d" % config)


def test_segments_edge_cases(dq8):
    rng = np.random.Generator(np.random.PCG64(4242))
    x = (rng.standard_normal(70000) * np.exp(rng.uniform(-6, 2, 70000))).astype(np.float32)
    x[rng.random(70000) < 0.05] = 0.0
    cases = [
        ("one segment", [0, 70000]),
        ("empty segments everywhere", [0, 0, 0, 5, 5, 1024, 1024, 1024, 2048, 30000, 30000, 70000, 70000]),
        ("tiny segments", list(range(0, 200)) + [70000]),
        ("ends inside quads and units", [0, 1, 3, 1023, 1025, 4097, 8190, 8193, 50001, 69999, 70000]),
        ("whole units", list(range(0, 70000, 1024)) + [70000]),
    ]
    for tag, b in cases:
        for kind in (0, 3):
            check_segments(dq8, kind, x, b, tag=tag)
    check_segments(dq8, 0, x, cases[3][1], x_off=1, c_off=3, tag="misaligned")
    check_segments(dq8, 1, x[:7], [0, 2, 7], tag="seven elements")
    zeros = np.zeros(5000, np.float32)
    zeros[4000:] = -0.0
    check_segments(dq8, 2, zeros, [0, 100, 4500, 5000], tag="all zero")


@pytest.mark.parametrize("seed", range(4))
def test_segments_random(dq8, seed):
    """Random cuts, among them the largest number of segments a call takes, over an array in which every wavefront
    walks several units."""
    rng = np.random.Generator(np.random.PCG64(5100 + seed))
    n = int(rng.integers(1_200_000, 2_500_000))
    n_seg = [4095, 1, 64, 700][seed]
    cuts = np.sort(rng.integers(0, n + 1, n_seg - 1)) if seed != 2 else np.sort(rng.integers(0, n // 50, n_seg - 1))
    bounds = np.concatenate([[0], cuts, [n]])
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-9, 2, n))).astype(np.float32)
    check_segments(dq8, int(rng.integers(0, 4)), x, bounds, x_off=int(seed == 3), tag="random %d" % seed)


def test_segment_calls_reject_bad_arguments(dq8):
    x = torch.zeros(100, device="cuda")
    with pytest.raises(dq8.Dq8Error, match="segments outside"):
        dq8.encode_segments(0, x, bounds_dev(np.arange(4098) % 101))
    with pytest.raises(ValueError):
        dq8.encode_segments(0, x, bounds_dev([0]))
    # offsets that do not ascend or lie beyond the array: no error is promised, but nothing outside the arrays is touched
    gc, gs = Guarded(100, np.uint8), Guarded(4, np.float32)
    dq8.encode_segments(0, dev(np.ones(100, np.float32)), bounds_dev([0, 90, 20, 10 ** 12, 100]), scales=gs.t, codes=gc.t)
    torch.cuda.synchronize()
    gc.check("malformed bounds")
    gs.check("malformed bounds")


@pytest.mark.parametrize("kind,K,with_local", [(0, 1, False), (0, 8, False), (1, 3, True), (2, 7, False), (3, 5, True),
                                               (0, 0, True), (0, 32, False)])
def test_average_of_segments(dq8, kind, K, with_local):
    """K workers' codes of tensors back to back, one scale per tensor and worker (the convnet's gradient set and an
    array cut at awkward places), averaged in one call: equal to the average of every tensor by itself."""
    rng = np.random.Generator(np.random.PCG64(6100 + 10 * K + kind))
    sizes = [t.size for _, t in workloads.tensors(2)]
    layouts = [(np.concatenate([[0], np.cumsum(sizes)]), 0, "C2"),
               (np.array([0, 0, 3, 1023, 1025, 4097, 9000, 9000, 20001, 33333]), 0, "awkward"),
               (np.array([0, 5000, 12000]), 1, "misaligned")]
    for bounds, off, tag in layouts:
        n, n_seg = int(bounds[-1]), len(bounds) - 1
        print("segment average %s kind=%d K=%d local=%d n=%d" % (tag, kind, K, with_local, n), flush=True)
        cl = [rng.integers(0, 256, n).astype(np.uint8) for _ in range(K)]
        sl = [np.exp(rng.uniform(-8, 8, n_seg)).astype(np.float32) for _ in range(K)]
        local = (rng.standard_normal(n) * np.exp(rng.uniform(-8, 8, n))).astype(np.float32) if with_local else None
        want = oracle.decode_accumulate_avg_segments(kind, cl, sl, bounds, local=local)
        go = Guarded(n, np.float32, off)
        dq8.decode_accumulate_avg_segments(kind, [dev(c, off) for c in cl], [dev(s) for s in sl], bounds_dev(bounds), out=go.t,
                                           local=None if local is None else dev(local, off))
        same_bits(go.t, want, "segment average " + tag)
        go.check("segment average " + tag)
