"""Pins for the oracle's projection, Eq.(1) (Sec. 2.2, 2.4, 3.1): g = R x."""
import numpy as np
import pytest
import torch

import oracle


def _dense_R(seed, kind, k, d, d_offset=0):
    return np.array([[oracle.r_entry(seed, kind, m, d_offset + j) for j in range(d)]
                     for m in range(k)])


@pytest.mark.parametrize("kind", [oracle.RADEMACHER, oracle.GAUSSIAN])
def test_projection_is_the_dense_matrix_product(kind):
    rng = np.random.default_rng(0)
    n, d, k = 5, 200, 64          # d not a multiple of 32: ragged last word
    G = rng.standard_normal((n, d)).astype(np.float32)
    R = _dense_R(7, kind, k, d)
    ref = G.astype(np.float64) @ R.T                 # library routine on a materialised R
    P = oracle.project(G, k, kind=kind, seed=7)
    np.testing.assert_allclose(P, ref.astype(np.float32), rtol=3e-7, atol=1e-6)
    # row sampler agrees and is fp64
    rows = [3, 0, 63]
    Pr = oracle.project_rows(G, rows, kind=kind, seed=7)
    np.testing.assert_allclose(Pr, ref[:, rows], rtol=1e-14, atol=1e-12)


def test_projection_brute_force_python():
    # third implementation: Python floats and explicit loops, tiny size
    rng = np.random.default_rng(1)
    n, d, k = 2, 64, 64
    G = rng.standard_normal((n, d)).astype(np.float32)
    P = oracle.project(G, k, seed=11)
    for i in range(n):
        for m in (0, 17, 63):
            acc = 0.0
            for j in range(d):
                acc += oracle.r_entry(11, 0, m, j) * float(G[i, j])
            assert np.float32(acc) == P[i, m]


def test_column_offset_splits_the_sum():
    rng = np.random.default_rng(2)
    n, d, k, a = 3, 512, 64, 160      # offset must keep whole 32-column words together
    G = rng.standard_normal((n, d)).astype(np.float32)
    whole = oracle.project_rows(G, range(k), seed=5)
    left = oracle.project_rows(G[:, :a], range(k), seed=5)
    right = oracle.project_rows(np.ascontiguousarray(G[:, a:]), range(k), seed=5, d_offset=a)
    np.testing.assert_allclose(whole, left + right, rtol=1e-13, atol=1e-11)
    # accumulate form: P += second slice
    P1 = oracle.project(G[:, :a], k, seed=5)
    P2 = oracle.project(np.ascontiguousarray(G[:, a:]), k, seed=5, d_offset=a, P=P1)
    np.testing.assert_allclose(P2, (P1.astype(np.float64) + right).astype(np.float32), rtol=0, atol=0)


def test_bf16_input_is_taken_at_its_stored_value():
    g = torch.Generator().manual_seed(3)
    Gb = torch.randn(4, 256, generator=g).to(torch.bfloat16)
    Pb = oracle.project(Gb, 64, seed=1)
    Pf = oracle.project(Gb.float().numpy(), 64, seed=1)
    np.testing.assert_array_equal(Pb, Pf)


def test_linearity_and_zero():
    rng = np.random.default_rng(4)
    G = rng.standard_normal((2, 320)).astype(np.float32)
    G3 = np.stack([G[0], G[1], np.zeros(320, np.float32)])
    P = oracle.project_rows(G3, range(64), seed=2)
    S = oracle.project_rows((G[0:1].astype(np.float64) * 2).astype(np.float32), range(64), seed=2)
    np.testing.assert_allclose(S[0], 2 * P[0], rtol=1e-14)
    assert np.all(P[2] == 0)


@pytest.mark.parametrize("kind,var", [(oracle.RADEMACHER, 1.0), (oracle.GAUSSIAN, None)])
def test_johnson_lindenstrauss_norms_and_inner_products(kind, var):
    # E|Rx|^2 = k * var(R) * |x|^2 ; relative spread sqrt(2/k) (Sec. 2.2: JL lemma)
    if var is None:
        var = oracle.gauss_table().var()
    rng = np.random.default_rng(5)
    n, d, k = 6, 4096, 1024
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[1] = 0.6 * G[0] + 0.8 * G[1]                    # cosine ~0.6 with row 0
    P = oracle.project_rows(G, range(k), kind=kind, seed=123)
    G64 = G.astype(np.float64)
    ratio = (P ** 2).sum(1) / (k * var * (G64 ** 2).sum(1))
    assert np.all(np.abs(ratio - 1) < 5 * np.sqrt(2.0 / k))
    cos_p = P[0] @ P[1] / np.linalg.norm(P[0]) / np.linalg.norm(P[1])
    cos_g = G64[0] @ G64[1] / np.linalg.norm(G64[0]) / np.linalg.norm(G64[1])
    assert abs(cos_p - cos_g) < 5 / np.sqrt(k)


def test_bad_arguments_are_refused():
    G = np.zeros((2, 64), np.float32)
    with pytest.raises(ValueError):
        oracle.project(G, 0)
    with pytest.raises(TypeError):
        oracle.project(G.astype(np.float64), 64)
