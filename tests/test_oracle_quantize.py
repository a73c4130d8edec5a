"""Pins for the oracle's quantiser, Eq.(4),(5) (Sec. 2.3, 3.1) and the 1-bit sign code
(Table 3 "Sign / 1-bit"; Sec. 5: the 1-bit representation has no zero bin)."""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.stats import norm

import oracle

BITS = [8, 4, 2, 1]


def _rne_fraction(x):
    """round-half-to-even of an exact rational"""
    f = x.numerator // x.denominator
    r = x - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_literal_formula_by_exact_rational_arithmetic(bits):
    rng = np.random.default_rng(bits)
    P = rng.standard_normal((3, 64)).astype(np.float32)
    q, S = oracle.quantize_unpacked(P, bits, literal=True)
    alpha = 2 ** (bits - 1) - 1
    for i in range(3):
        Sx = max(abs(Fraction(float(v))) for v in P[i])
        assert Fraction(float(S[i])) == Sx
        for m in range(64):
            # fp64 evaluation of alpha*x/S is within 2^-50 of the rational value; no entry of this
            # sample sits that close to a half-integer, so the exact rounding must agree
            assert q[i, m] == _rne_fraction(alpha * Fraction(float(P[i, m])) / Sx)


def test_round_half_to_even_hand_cases():
    # bits=4: alpha = 7; with S = 7 the code is rne(x) itself
    x = np.zeros((1, 64), np.float32)
    x[0, :8] = [7.0, 0.5, 1.5, 2.5, -2.5, -0.5, 3.5, -3.5]
    for literal in (False, True):
        q, S = oracle.quantize_unpacked(x, 4, literal=literal)
        assert S[0] == 7.0
        assert list(q[0, :8]) == [7, 0, 2, 2, -2, 0, 4, -4]
    # bits=2: alpha = 1: |x| < S/2 -> 0, exactly S/2 -> 0 (tie to even), above -> +-1
    y = np.zeros((1, 64), np.float32)
    y[0, :6] = [4.0, 2.0, -2.0, 2.0000002, -3.0, 1.9999999]
    q, _ = oracle.quantize_unpacked(y, 2)
    assert list(q[0, :6]) == [1, 0, 0, 1, -1, 0]


@pytest.mark.parametrize("bits", BITS)
def test_code_range_extreme_element_and_packing(bits):
    rng = np.random.default_rng(10 + bits)
    n, k = 7, 256
    P = (rng.standard_normal((n, k)) * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)
    codes, S, rn = oracle.quantize(P, bits)
    assert codes.shape == (n, k * bits // 8) and codes.dtype == np.uint8
    q = oracle.unpack(codes, k, bits)
    qu, Su = oracle.quantize_unpacked(P, bits)
    np.testing.assert_array_equal(q, qu)
    np.testing.assert_array_equal(S, np.abs(P).max(1))
    alpha = max(2 ** (bits - 1) - 1, 1)
    assert q.min() >= -alpha and q.max() <= alpha
    if bits == 1:
        assert set(np.unique(q)) == {-1, 1}
        np.testing.assert_array_equal(q, np.where(P < 0, -1, 1))
    else:
        am = np.abs(P).argmax(1)
        assert np.all(np.abs(q[np.arange(n), am]) == alpha)
    n2 = (q.astype(np.int64) ** 2).sum(1)
    np.testing.assert_array_equal(rn, (1.0 / np.sqrt(n2.astype(np.float64))).astype(np.float32))
    np.testing.assert_array_equal(oracle.pack(q, bits), codes)


def test_packed_layout_by_hand():
    k = 64
    q = np.zeros((1, k), np.int8)
    q[0, :6] = [1, -1, 0, -7, 7, -3]
    c8 = oracle.pack(q, 8)[0]
    assert list(c8[:6]) == [1, 255, 0, 249, 7, 253]
    c4 = oracle.pack(q, 4)[0]           # element 2t in the low nibble, 2t+1 in the high nibble
    assert list(c4[:3]) == [0x1 | (0xF << 4), 0x0 | (0x9 << 4), 0x7 | (0xD << 4)]
    t = np.zeros((1, k), np.int8)
    t[0, [0, 1, 9, 63]] = [1, -1, -1, 1]
    c2 = oracle.pack(t, 2)[0]           # plane "non-zero" then plane "negative"
    assert c2.size == 16
    assert c2[0] == 0b11 and c2[1] == 0b10 and c2[7] == 0x80
    assert c2[8] == 0b10 and c2[9] == 0b10 and c2[15] == 0
    s = np.ones((1, k), np.int8)
    s[0, [0, 8, 63]] = -1
    c1 = oracle.pack(s, 1)[0]
    assert c1.size == 8 and c1[0] == 1 and c1[1] == 1 and c1[7] == 0x80 and c1[2] == 0


@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_scale_invariance(bits):
    rng = np.random.default_rng(20 + bits)
    P = rng.standard_normal((4, 128)).astype(np.float32)
    c0, S0, r0 = oracle.quantize(P, bits)
    for p in (-20, 3, 40):
        c, S, r = oracle.quantize(P * np.float32(2.0 ** p), bits)
        np.testing.assert_array_equal(c, c0)
        np.testing.assert_array_equal(S, S0 * np.float32(2.0 ** p))
        np.testing.assert_array_equal(r, r0)


@pytest.mark.parametrize("bits", BITS)
def test_zero_vector_and_signed_zero(bits):
    P = np.zeros((2, 64), np.float32)
    P[1, 0] = -0.0
    P[1, 1] = 1.0
    P[1, 2] = -1.0
    codes, S, rn = oracle.quantize(P, bits)
    q = oracle.unpack(codes, 64, bits)
    assert S[0] == 0
    if bits == 1:
        assert np.all(q[0] == 1) and rn[0] == np.float32(1 / 8.0)
        assert q[1, 0] == 1 and q[1, 1] == 1 and q[1, 2] == -1     # -0.0 is not negative
    else:
        assert np.all(q[0] == 0) and rn[0] == 0


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_canonical_fp32_codes_differ_from_literal_only_on_rounding_boundaries(bits):
    rng = np.random.default_rng(30 + bits)
    P = rng.standard_normal((64, 8192)).astype(np.float32)
    qc, S = oracle.quantize_unpacked(P, bits)
    ql, _ = oracle.quantize_unpacked(P, bits, literal=True)
    diff = qc != ql
    assert diff.mean() <= 1e-4
    if diff.any():
        assert np.abs(qc.astype(int) - ql.astype(int))[diff].max() == 1
        alpha = 2 ** (bits - 1) - 1
        x = alpha * P.astype(np.float64) / S[:, None].astype(np.float64)
        frac = np.abs(x - np.floor(x) - 0.5)
        assert frac[diff].max() < 1e-4


def test_zero_bin_occupancy_matches_the_normal_law():
    # Sec. 5: under absmax scaling most Gaussian-like entries fall into the zero bin at 2 and 4
    # bits; 1-bit has no zero bin.  Given the realised S the expected share is 2*Phi(S/(2 alpha))-1.
    rng = np.random.default_rng(40)
    P = rng.standard_normal((32, 8192)).astype(np.float32)
    for bits in (8, 4, 2):
        q, S = oracle.quantize_unpacked(P, bits)
        alpha = 2 ** (bits - 1) - 1
        expect = (2 * norm.cdf(S / (2.0 * alpha)) - 1).mean()
        got = (q == 0).mean()
        assert abs(got - expect) < 0.01
    q2, _ = oracle.quantize_unpacked(P, 2)
    q4, _ = oracle.quantize_unpacked(P, 4)
    q8, _ = oracle.quantize_unpacked(P, 8)
    q1, _ = oracle.quantize_unpacked(P, 1)
    assert (q2 == 0).mean() > 0.9 and 0.15 < (q4 == 0).mean() < 0.3 and (q8 == 0).mean() < 0.02
    assert (q1 == 0).mean() == 0


def test_storage_column_of_table_1():
    """N k C b / 8 bytes reproduces the paper's storage column (GiB) for ~270K examples."""
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_storage.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    table = {int(b): float(gb) for b, gb in rows}
    N, k, C = 270_000, 8192, 4
    for bits, gb in table.items():
        size = N * C * (oracle.code_bytes(k, bits) if bits != 16 else 2 * k)
        assert abs(size / 2 ** 30 - gb) / gb < 0.01
    assert table[16] / table[1] == pytest.approx(16, rel=0.005)      # "up to 16x" (abstract)
    for bits in (8, 4, 2, 1):
        assert oracle.code_bytes(k, bits) * 16 == 2 * k * bits
