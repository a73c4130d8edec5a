"""Pins for the oracle's mixed-precision influence: b-bit train codes (paper Sec. 3.1, Eq.(4),(5)) scored
against validation gradients kept at 16 bits as in LESS (Sec. 2.2, Eq.(2)), combined as in Eq.(7).
The paper quantises both sides alike; the variant is this build's, so it is pinned by brute force and by
the cases in which it must coincide with the other, independently pinned, scoring functions."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _bf16_to_f64(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _rows(n, k, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, k)) * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)


@pytest.mark.parametrize("bits", [8, 4, 2, 1])
def test_brute_force_with_exact_rationals(bits):
    """Tiny case, every product and sum as exact rationals of the stored values."""
    C, N, M, k = 2, 5, 3, 64
    eta = [1.0, 0.375]
    tq = [oracle.quantize(_rows(N, k, 30 + c), bits) for c in range(C)]
    va = [oracle.less16_store(_rows(M, k, 40 + c)) for c in range(C)]
    sc, full = oracle.score_mixed([t[0] for t in tq], [t[2] for t in tq], va, eta, k, bits, want_full=True)
    for z in range(N):
        for v in range(M):
            acc = Fraction(0)
            for c in range(C):
                q = oracle.unpack(tq[c][0][z:z + 1], k, bits)[0]
                y = _bf16_to_f64(va[c][v])
                d = sum(Fraction(int(q[m])) * Fraction(float(y[m])) for m in range(k))
                acc += Fraction(float(np.float32(eta[c]))) * Fraction(float(tq[c][2][z])) * d
            assert abs(full[z, v] - float(acc)) <= 1e-12 * max(1.0, abs(float(acc)))
        assert sc[z] == full[z].max()


@pytest.mark.parametrize("bits", [8, 4, 2, 1])
def test_equals_numpy_matrix_product_of_the_stored_values(bits):
    C, N, M, k = 3, 40, 9, 256
    eta = [1.0, 0.5, 0.25]
    tq = [oracle.quantize(_rows(N, k, 50 + c), bits) for c in range(C)]
    va = [oracle.less16_store(_rows(M, k, 60 + c)) for c in range(C)]
    sc, full = oracle.score_mixed([t[0] for t in tq], [t[2] for t in tq], va, eta, k, bits, want_full=True)
    ref = np.zeros((N, M))
    for c in range(C):
        q = oracle.unpack(tq[c][0], k, bits).astype(np.float64)
        ref += eta[c] * tq[c][2].astype(np.float64)[:, None] * (q @ _bf16_to_f64(va[c]).T)
    np.testing.assert_allclose(full, ref, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(sc, full.max(axis=1))


@pytest.mark.parametrize("bits", [8, 4, 2, 1])
def test_coincides_with_the_quantised_score_when_validation_rows_are_scaled_codes(bits):
    """Validation rows that are themselves code vectors times 2^-7 are exact in bfloat16 (|q| <= 127 has 7
    bits): the mixed influence is then Eq.(7) with 2^-7 in place of the validation norm factor."""
    C, N, M, k = 2, 30, 6, 128
    eta = [1.0, 0.5]
    tq = [oracle.quantize(_rows(N, k, 70 + c), bits) for c in range(C)]
    vq = [oracle.quantize(_rows(M, k, 80 + c), bits) for c in range(C)]
    v16 = []
    for c in range(C):
        vals = (oracle.unpack(vq[c][0], k, bits).astype(np.float32) * np.float32(2.0 ** -7))
        u = vals.view(np.uint32)
        assert not (u & 0xFFFF).any()                                        # exactly representable
        v16.append((u >> 16).astype(np.uint16))
    sc_m, full_m = oracle.score_mixed([t[0] for t in tq], [t[2] for t in tq], v16, eta, k, bits, want_full=True)
    vr = [np.full(M, 2.0 ** -7, dtype=np.float32) for _ in range(C)]
    sc_q, full_q = oracle.score([t[0] for t in tq], [t[2] for t in tq], [v[0] for v in vq], vr, eta, k, bits, want_full=True)
    np.testing.assert_allclose(full_m, full_q.astype(np.float64), rtol=3e-7, atol=1e-9)   # fp32 epilogue of oracle.score


def test_approaches_the_16_bit_cosine_as_the_train_codes_get_finer():
    """With 8-bit train codes the mixed influence is close to the all-16-bit LESS cosine of the same vectors
    (Eq.(3)), and closer than the 2-bit codes' (the point of keeping more bits)."""
    C, N, M, k = 1, 64, 8, 2048
    P, V = _rows(N, k, 90), _rows(M, k, 91)
    V[:4] = 0.6 * P[:4] / np.linalg.norm(P[:4], axis=1, keepdims=True) * np.linalg.norm(V[:4], axis=1, keepdims=True) + 0.8 * V[:4]
    t16, v16 = oracle.less16_store(P), oracle.less16_store(V)
    ref = oracle.less16_score([t16], [v16], [1.0], want_full=True)[1]
    err = {}
    for bits in (8, 2):
        c, _, rn = oracle.quantize(P, bits)
        full = oracle.score_mixed([c], [rn], [v16], [1.0], k, bits, want_full=True)[1]
        err[bits] = np.abs(full - ref).max()
    assert err[8] < 5e-3 and err[8] < err[2]


def test_linear_in_eta_and_zero_code_rows_score_zero():
    C, N, M, k = 2, 10, 4, 64
    tq = [oracle.quantize(_rows(N, k, 95 + c), 4) for c in range(C)]
    for c in range(C):
        tq[c][0][3] = 0
        tq[c][2][3] = 0.0
    va = [oracle.less16_store(_rows(M, k, 97 + c)) for c in range(C)]
    f = lambda eta: oracle.score_mixed([t[0] for t in tq], [t[2] for t in tq], va, eta, k, 4, want_full=True)[1]
    np.testing.assert_allclose(f([1.0, 0.5]), f([1.0, 0.0]) + f([0.0, 0.5]), atol=1e-13)
    assert not f([1.0, 0.5])[3].any()
