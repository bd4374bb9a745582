"""Pins for the oracle's codebooks (Sec. 3.1 of arXiv 1511.04561).

The oracle evaluates closed-form integer ratios; these tests reach the same tables
by other routes: reading the bits of each pattern and walking the bisection tree in
exact rational arithmetic, and the structural facts the paper states.
"""
import hashlib
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.exact import codebook_exact, round_to_f32

KINDS = [oracle.DYNAMIC_TREE, oracle.LINEAR, oracle.STATIC_TREE]


@pytest.mark.parametrize("kind", KINDS + [oracle.MANTISSA])
def test_tree_walk_in_exact_rationals_gives_the_same_table(kind):
    cb = oracle.codebook(kind)
    exact = codebook_exact(kind)
    for c in range(256):
        want = round_to_f32(exact[c])
        if c >= 128 and exact[c] == 0:
            want = np.float32(-0.0)
        assert cb[c].view(np.uint32) == np.float32(want).view(np.uint32), (kind, c, cb[c], want)


@pytest.mark.parametrize("kind", KINDS)
def test_sign_symmetry_and_monotonicity(kind):
    cb = oracle.codebook(kind)
    bits = cb.view(np.uint32)
    assert cb.shape == (256,) and cb.dtype == np.float32
    assert np.all(bits[128:] == (bits[:128] | np.uint32(0x80000000)))  # code bit 7 is the sign
    assert np.all(np.diff(cb[:128].astype(np.float64)) > 0)  # 128 distinct ascending magnitudes
    assert np.all(cb[:128] >= 0) and np.all(cb[:128] <= 1)


def test_dynamic_tree_structure():
    cb = oracle.codebook(oracle.DYNAMIC_TREE).astype(np.float64)
    assert cb[0] == 0.0  # the pattern without a flag bit
    # n leading zeros -> decade 10^-n; 2^(6-n) tree leaves inside the open interval (0.1, 1) * 10^-n
    for n in range(7):
        lo, hi = 0.1 * 10.0 ** -n, 1.0 * 10.0 ** -n
        inside = np.sum((cb[:128] > lo) & (cb[:128] < hi))
        assert inside == 2 ** (6 - n), (n, inside)
    assert 64 + 32 + 16 + 8 + 4 + 2 + 1 + 1 == 128
    # largest exponent is 10^-6: the smallest non-zero value lies in (1e-7, 1e-6), nothing below
    assert 1e-7 < cb[1] < 1e-6
    assert abs(cb[1] - 5.5e-7) < 1e-13  # middle of (0.1, 1) * 1e-6
    # equal leaf width inside a decade (bisection into equal pieces)
    top = cb[64:128]
    assert np.allclose(np.diff(top), 0.9 / 64, rtol=0, atol=1e-7)
    assert abs(top[0] - (0.1 + 0.45 / 64)) < 1e-7 and abs(top[-1] - (1 - 0.45 / 64)) < 1e-7


def test_linear_structure():
    cb = oracle.codebook(oracle.LINEAR)
    assert cb[0] == 0.0 and cb[127] == 1.0
    assert np.allclose(np.diff(cb[:128].astype(np.float64)), 1.0 / 127.0, rtol=0, atol=1e-7)


def test_static_tree_structure():
    cb = oracle.codebook(oracle.STATIC_TREE).astype(np.float64)
    for e in range(8):  # 3 exponent bits -> 8 decades, 4 tree bits -> 16 leaves each
        lo, hi = 0.1 * 10.0 ** (e - 7), 1.0 * 10.0 ** (e - 7)
        dec = cb[16 * e:16 * e + 16]
        assert np.all((dec > lo) & (dec < hi))
        assert np.allclose(np.diff(dec), 0.9 / 16 * 10.0 ** (e - 7), rtol=1e-5, atol=0)
    assert np.all(cb[:128] > 0)  # this type has no zero
    assert abs(cb[127] - 0.971875) < 1e-7


def test_mantissa_structure():
    """Sec. 3.1: a 3-bit exponent and a mantissa that holds 0..15.  The type repeats values: zero once per
    exponent, and ten tenths of a decade are one tenth of the next."""
    cb = oracle.codebook(oracle.MANTISSA)
    bits = cb.view(np.uint32)
    assert np.all(bits[128:] == (bits[:128] | np.uint32(0x80000000)))
    mags = cb[:128]
    for E in range(8):
        dec = mags[16 * E:16 * E + 16].astype(np.float64)
        assert dec[0] == 0
        assert np.allclose(dec[1:] / dec[1], np.arange(1, 16), rtol=1e-6)  # equal steps: a linear mantissa
        if E < 7:
            assert mags[16 * E + 10] == mags[16 * (E + 1) + 1]  # 10 tenths = 1 tenth of the next decade
            assert mags[16 * E + 15] < mags[16 * (E + 1) + 2]
    assert mags[16 * 7 + 10] == 1.0 and mags.max() == np.float32(1.5)
    assert float(mags[1]) == float(np.float32(1e-8))
    assert len(set(mags.tolist())) == 1 + 8 * 15 - 7  # 114 distinct magnitudes


def test_paper_worked_examples_fall_in_the_oracle_leaf(golden_dir):
    """Sec. 3.1 prints approximations of two numbers; each must share a tree leaf with the input."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "worked_examples.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 2
    cb = oracle.codebook(oracle.DYNAMIC_TREE)
    for x_txt, approx_txt in rows:
        x, approx = Fraction(x_txt), Fraction(approx_txt)
        n = 0
        while x < Fraction(1, 10 ** (n + 1)):
            n += 1
        t = 6 - n
        width = Fraction(9, 10) / 2 ** t / 10 ** n
        k = int((x - Fraction(1, 10 ** (n + 1))) / width)
        lo = Fraction(1, 10 ** (n + 1)) + k * width
        assert lo < x < lo + width and lo < approx < lo + width
        # the oracle's code for x (scale 1) is the middle of that same leaf
        codes, _ = oracle.encode(oracle.DYNAMIC_TREE, np.array([float(x)], np.float32), 0,
                                 scales=np.ones(1, np.float32))
        v = Fraction(float(cb[codes[0]]))
        assert lo < v < lo + width
        assert abs(v - (lo + width / 2)) < (lo + width / 2) * Fraction(1, 10 ** 7)  # fp32 rounding


def test_regression_hashes(golden_dir):
    want = dict(l.split() for l in open(os.path.join(golden_dir, "codebook_sha256.txt")) if l[0] != "#")
    for kind in KINDS + [oracle.MANTISSA]:
        assert hashlib.sha256(oracle.codebook(kind).astype("<f4").tobytes()).hexdigest() == want[str(kind)]


def test_bad_kind_is_an_error():
    with pytest.raises(ValueError):
        oracle.codebook(7)
