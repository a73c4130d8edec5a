"""Pins for the oracle's absmean quantiser variant (paper Sec. 5, Table 3).

The paper prints no formula for the absmean scheme, so the rule itself (BitNet-style
q = clamp(rne(g / mean|g|), -alpha, alpha)) is this build's reading: PARITY UNPINNED against the
paper.  What is pinned here is that the oracle computes exactly that rule: against numpy's own
IEEE float32 arithmetic, against exact rational arithmetic for the fixed-point mean, by the
invariances the rule must have, and by the one qualitative fact the paper states (the zero bin
that absmax fills at low widths is emptied)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _rows(n, k, seed, spread=True):
    rng = np.random.default_rng(seed)
    P = rng.standard_normal((n, k))
    if spread:
        P *= np.exp(rng.standard_normal((n, 1)))
    return P.astype(np.float32)


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_codes_follow_the_rule_in_numpy_float32(bits):
    P = _rows(16, 256, 1)
    codes, S, rn, q = oracle.quantize_absmean(P, bits, want_unpacked=True)
    alpha = 2 ** (bits - 1) - 1
    np.testing.assert_allclose(S, np.abs(P.astype(np.float64)).mean(1), rtol=2e-7)
    scale = (np.float32(1.0) / S).astype(np.float32)
    want = np.clip(np.rint((P * scale[:, None]).astype(np.float32)), -alpha, alpha).astype(np.int8)
    np.testing.assert_array_equal(q, want)
    np.testing.assert_array_equal(oracle.unpack(codes, 256, bits), want)
    n2 = (want.astype(np.int64) ** 2).sum(1)
    np.testing.assert_array_equal(rn, (1.0 / np.sqrt(n2.astype(np.float64))).astype(np.float32))


def test_mean_is_the_fixed_point_mean_exactly():
    P = _rows(6, 64, 2)
    P[3, 5] = 1e-12          # far below the maximum: truncated by the fixed point, not lost silently
    _, S, _ = oracle.quantize_absmean(P, 4)
    for i in range(P.shape[0]):
        A = float(np.abs(P[i]).max())
        _, E = math.frexp(A)
        U = sum(int(Fraction(float(abs(x))) * Fraction(2) ** (32 - E)) for x in P[i])   # exact truncation
        want = np.float32(math.ldexp(float(U) / float(P.shape[1]), E - 32))
        assert S[i] == want
        exact = sum(Fraction(float(abs(x))) for x in P[i]) / P.shape[1]
        assert abs(Fraction(float(S[i])) - exact) <= exact * Fraction(1, 2 ** 22)


def test_order_of_elements_does_not_change_the_scale():
    P = _rows(4, 1024, 3)
    perm = np.random.default_rng(0).permutation(1024)
    c1, S1, r1, q1 = oracle.quantize_absmean(P, 4, want_unpacked=True)
    c2, S2, r2, q2 = oracle.quantize_absmean(P[:, perm], 4, want_unpacked=True)
    np.testing.assert_array_equal(S1, S2)
    np.testing.assert_array_equal(q1[:, perm], q2)
    np.testing.assert_array_equal(r1, r2)


@pytest.mark.parametrize("bits", [8, 4, 2, 1])
def test_power_of_two_scaling_and_negation(bits):
    P = _rows(8, 256, 4)
    c, S, r = oracle.quantize_absmean(P, bits)
    c2, S2, r2 = oracle.quantize_absmean(P * np.float32(8.0), bits)
    np.testing.assert_array_equal(c, c2)
    np.testing.assert_array_equal(S * np.float32(8.0), S2)
    qa = oracle.unpack(c, 256, bits)
    qn = oracle.unpack(oracle.quantize_absmean(-P, bits)[0], 256, bits)
    if bits > 1:
        np.testing.assert_array_equal(qn, -qa)
    else:
        np.testing.assert_array_equal(qn[P != 0], -qa[P != 0])


def test_one_bit_is_the_sign_code_and_zero_rows():
    P = _rows(5, 128, 5)
    P[2] = 0.0
    c, S, r = oracle.quantize_absmean(P, 1)
    c0, _, r0 = oracle.quantize(P, 1)
    np.testing.assert_array_equal(c, c0)
    np.testing.assert_array_equal(r, r0)
    assert S[2] == 0.0 and S[0] > 0
    c4, S4, r4 = oracle.quantize_absmean(P, 4)
    assert S4[2] == 0.0 and r4[2] == 0.0 and not c4[2].any()


def test_zero_bin_is_emptied_relative_to_absmax():
    """Sec. 5: absmax puts most entries of a low-width code in the zero bin, the mean-based scale does
    not.  For Gaussian entries P(q = 0) = P(|g| < mean|g| / 2) = erf(sqrt(2/pi) / (2 sqrt 2))."""
    k = 8192
    P = _rows(32, k, 6, spread=False)
    _, _, _, qm = oracle.quantize_absmean(P, 2, want_unpacked=True)
    qx, _ = oracle.quantize_unpacked(P, 2)
    zero_mean = (qm == 0).mean()
    zero_max = (qx == 0).mean()
    assert abs(zero_mean - math.erf(math.sqrt(2 / math.pi) / (2 * math.sqrt(2)))) < 5e-3
    assert zero_max > 0.9 and zero_mean < 0.35
    # and the higher widths lose range instead (Sec. 5: "at the cost of reducing the fidelity"):
    _, _, _, q8 = oracle.quantize_absmean(P, 8, want_unpacked=True)
    assert np.abs(q8).max() <= 6          # a Gaussian reaches ~5 mean-absolute-deviations: 6 of 127 levels used
