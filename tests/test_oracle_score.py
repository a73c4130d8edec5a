"""Pins for the oracle's influence score, Eq.(6),(7) (Sec. 3.2), the max over validation
vectors, and the selection rule of Sec. 4.1."""
import numpy as np
import pytest

import oracle

BITS = [8, 4, 2, 1]


def _store(rng, n, k, bits, C):
    P = [rng.standard_normal((n, k)).astype(np.float32) for _ in range(C)]
    out = [oracle.quantize(p, bits) for p in P]
    return P, [o[0] for o in out], [o[2] for o in out]


@pytest.mark.parametrize("bits", BITS)
def test_brute_force_python_integers(bits):
    rng = np.random.default_rng(bits)
    N, M, k, C = 4, 2, 64, 2
    _, tc, tr = _store(rng, N, k, bits, C)
    _, vc, vr = _store(rng, M, k, bits, C)
    eta = [0.7, 0.2]
    sc, full = oracle.score(tc, tr, vc, vr, eta, k, bits, want_full=True)
    tq = [oracle.unpack(c, k, bits) for c in tc]
    vq = [oracle.unpack(c, k, bits) for c in vc]
    for z in range(N):
        best = None
        for v in range(M):
            acc = np.float32(0)
            exact = 0.0
            for i in range(C):
                D = sum(int(a) * int(b) for a, b in zip(tq[i][z], vq[i][v]))
                w = np.float32(eta[i]) * vr[i][v]
                t = np.float32(np.float32(D) * tr[i][z]) * w
                acc = np.float32(acc + t)
                na = np.sqrt(float(sum(int(a) ** 2 for a in tq[i][z])))
                nb = np.sqrt(float(sum(int(b) ** 2 for b in vq[i][v])))
                exact += eta[i] * D / (na * nb)
            assert full[z, v] == acc
            assert abs(float(acc) - exact) < 1e-6         # it is the cosine sum of Eq.(7)
            best = acc if best is None or acc > best else best
        assert sc[z] == best


@pytest.mark.parametrize("bits", BITS)
def test_single_pair_is_numpy_cosine_of_codes(bits):
    rng = np.random.default_rng(50 + bits)
    k = 512
    _, tc, tr = _store(rng, 1, k, bits, 1)
    _, vc, vr = _store(rng, 1, k, bits, 1)
    sc = oracle.score(tc, tr, vc, vr, [1.0], k, bits)
    a = oracle.unpack(tc[0], k, bits)[0].astype(np.float64)
    b = oracle.unpack(vc[0], k, bits)[0].astype(np.float64)
    assert abs(sc[0] - a @ b / np.linalg.norm(a) / np.linalg.norm(b)) < 2e-7


@pytest.mark.parametrize("bits", BITS)
def test_self_similarity_is_one_and_negation_flips(bits):
    rng = np.random.default_rng(60 + bits)
    k, C = 1024, 3
    P, tc, tr = _store(rng, 6, k, bits, C)
    eta = [0.5, 0.25, 0.25]
    _, full = oracle.score(tc, tr, tc, tr, eta, k, bits, want_full=True)
    np.testing.assert_allclose(np.diag(full), 1.0, atol=4e-7)
    assert np.all(np.abs(full) <= 1 + 4e-7)                # |score| <= sum |eta|
    np.testing.assert_allclose(full, full.T, atol=3e-7)
    # negate train vectors: codes negate (no zeros in P), so every score changes sign
    neg = [oracle.quantize(-p, bits) for p in P]
    _, fneg = oracle.score([o[0] for o in neg], [o[2] for o in neg], tc, tr, eta, k, bits,
                           want_full=True)
    np.testing.assert_array_equal(fneg, -full)


def test_sign_code_dot_is_k_minus_twice_hamming():
    rng = np.random.default_rng(70)
    k = 2048
    _, tc, tr = _store(rng, 5, k, 1, 1)
    _, vc, vr = _store(rng, 3, k, 1, 1)
    _, full = oracle.score(tc, tr, vc, vr, [1.0], k, 1, want_full=True)
    for z in range(5):
        for v in range(3):
            ham = int(np.unpackbits(tc[0][z] ^ vc[0][v]).sum())
            assert full[z, v] == np.float32(np.float32(np.float32(k - 2 * ham) * tr[0][z]) * vr[0][v])
    assert np.all(tr[0] == np.float32(1 / np.sqrt(k)))


def test_two_bit_dot_from_bit_planes():
    rng = np.random.default_rng(71)
    k = 1024
    _, tc, _ = _store(rng, 3, k, 2, 1)
    _, vc, _ = _store(rng, 2, k, 2, 1)
    tq, vq = oracle.unpack(tc[0], k, 2), oracle.unpack(vc[0], k, 2)
    for z in range(3):
        for v in range(2):
            nza, sga = tc[0][z][:k // 8], tc[0][z][k // 8:]
            nzb, sgb = vc[0][v][:k // 8], vc[0][v][k // 8:]
            both = nza & nzb
            D = int(np.unpackbits(both).sum()) - 2 * int(np.unpackbits(both & (sga ^ sgb)).sum())
            assert D == int(tq[z].astype(int) @ vq[v].astype(int))


@pytest.mark.parametrize("bits", [8, 2])
def test_linearity_in_eta_zero_weight_and_row_permutation(bits):
    rng = np.random.default_rng(80 + bits)
    N, M, k, C = 16, 5, 256, 3
    _, tc, tr = _store(rng, N, k, bits, C)
    _, vc, vr = _store(rng, M, k, bits, C)
    eta = np.array([1.0, 0.5, 0.25], np.float32)
    sc, full = oracle.score(tc, tr, vc, vr, eta, k, bits, want_full=True)
    _, full2 = oracle.score(tc, tr, vc, vr, 2 * eta, k, bits, want_full=True)
    np.testing.assert_array_equal(full2, 2 * full)         # power-of-two factor: exact
    parts = [oracle.score([tc[i]], [tr[i]], [vc[i]], [vr[i]], [eta[i]], k, bits, want_full=True)[1]
             for i in range(C)]
    np.testing.assert_allclose(full, sum(p.astype(np.float64) for p in parts), atol=3e-7)
    # a checkpoint with zero weight changes nothing
    sc0 = oracle.score(tc + [tc[0]], tr + [tr[0]], vc + [vc[0]], vr + [vr[0]],
                       list(eta) + [0.0], k, bits)
    np.testing.assert_array_equal(sc0, sc)
    np.testing.assert_array_equal(sc, full.max(1))
    perm = rng.permutation(N)
    scp = oracle.score([c[perm] for c in tc], [r[perm] for r in tr], vc, vr, eta, k, bits)
    np.testing.assert_array_equal(scp, sc[perm])


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_scale_cancels_dequantised_cosine_equals_code_cosine(bits):
    # Sec. 4.1 says codes are "reconstructed, normalized"; Eq.(6) normalises codes directly.
    rng = np.random.default_rng(90 + bits)
    k = 512
    P = (rng.standard_normal((3, k)) * [[1.0], [1e-3], [1e4]]).astype(np.float32)
    codes, S, rn = oracle.quantize(P, bits)
    q = oracle.unpack(codes, k, bits).astype(np.float64)
    alpha = 2 ** (bits - 1) - 1
    deq = q * (S[:, None].astype(np.float64) / alpha)
    _, full = oracle.score([codes], [rn], [codes], [rn], [1.0], k, bits, want_full=True)
    cosd = (deq @ deq.T) / np.outer(np.linalg.norm(deq, axis=1), np.linalg.norm(deq, axis=1))
    np.testing.assert_allclose(full, cosd, atol=3e-7)


def test_sign_codes_follow_the_simhash_law():
    # binary quantised random projection (Sec. 2.4): E[<sign a, sign b>]/k = 1 - 2 arccos(rho)/pi
    rng = np.random.default_rng(100)
    k = 8192
    for rho in (0.0, 0.3, 0.5, 0.9):
        a = rng.standard_normal((1, k)).astype(np.float32)
        b = (rho * a + np.sqrt(1 - rho ** 2) * rng.standard_normal((1, k))).astype(np.float32)
        ca, _, ra = oracle.quantize(a, 1)
        cb, _, rb = oracle.quantize(b, 1)
        s = oracle.score([ca], [ra], [cb], [rb], [1.0], k, 1)[0]
        assert abs(s - (1 - 2 * np.arccos(rho) / np.pi)) < 4 / np.sqrt(k)


def test_more_bits_track_the_less_cosine_more_closely():
    rng = np.random.default_rng(110)
    N, M, k, C = 64, 8, 2048, 2
    tP = [rng.standard_normal((N, k)).astype(np.float32) for _ in range(C)]
    vP = [(0.5 * t[:M] + rng.standard_normal((M, k))).astype(np.float32) for t in tP]
    eta = [1.0, 0.5]
    less = oracle.less_cosine(tP, vP, eta)
    ref = sum(e * (t.astype(np.float64) / np.linalg.norm(t, axis=1, keepdims=True)) @
              (v.astype(np.float64) / np.linalg.norm(v, axis=1, keepdims=True)).T
              for e, t, v in zip(eta, tP, vP))
    np.testing.assert_allclose(less, ref, atol=1e-8)
    errs = []
    for bits in BITS:
        t = [oracle.quantize(p, bits) for p in tP]
        v = [oracle.quantize(p, bits) for p in vP]
        _, full = oracle.score([o[0] for o in t], [o[2] for o in t], [o[0] for o in v],
                               [o[2] for o in v], eta, k, bits, want_full=True)
        errs.append(np.abs(full - less).max())
    assert errs[0] < 0.01 and errs[0] < errs[1] < errs[2]
    # planted pairs (train z = val z for z < M) win the row maximum at every width
    assert np.all(less[:M].argmax(1) == np.arange(M))


def test_topk_against_lexsort_with_ties():
    rng = np.random.default_rng(120)
    s = rng.integers(-5, 5, size=1000).astype(np.float32) / 4        # many ties
    for k_sel in (0, 1, 50, 999, 1000):
        idx, val = oracle.topk(s, k_sel)
        ref = np.lexsort((np.arange(s.size), -s))[:k_sel]
        np.testing.assert_array_equal(idx, ref)
        np.testing.assert_array_equal(val, s[ref])
    s2 = np.array([0.0, -0.0, 1.0, -1.0, 1.0], np.float32)
    idx, _ = oracle.topk(s2, 5)
    assert list(idx) == [2, 4, 0, 1, 3]
    with pytest.raises(ValueError):
        oracle.topk(s, 1001)


def test_planted_pairs_are_recovered_tiny_config():
    """Config 1: 1024 train / 64 val vectors of dimension 16384, 32 planted pairs, k = 512,
    8-bit, top-50 must contain every planted train index."""
    import torch
    from paper_2502_01703_amd import synth
    train, val, planted = synth.config1()
    tP = oracle.project(train, 512, seed=0)
    vP = oracle.project(val, 512, seed=0)
    for bits, need in ((8, 32), (1, 30)):
        tc, _, tr = oracle.quantize(tP, bits)
        vc, _, vr = oracle.quantize(vP, bits)
        sc = oracle.score([tc], [tr], [vc], [vr], [1.0], 512, bits)
        idx, _ = oracle.topk(sc, 50)
        hit = len(set(idx.tolist()) & set(planted.tolist()))
        assert hit >= need, (bits, hit)
