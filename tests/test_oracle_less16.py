"""Pins for the oracle's 16-bit LESS comparator (paper Sec. 2.2, Eq.(2),(3); Table 1's baseline store).
"16-bit" is read as bfloat16 (the paper does not name the format)."""
import numpy as np
import torch

import oracle


def _bf16_to_f64(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _rows(n, k, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, k)) * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)


def test_store_is_the_rounded_unit_vector():
    P = _rows(12, 320, 1)
    P[4] = 0.0
    st = oracle.less16_store(P)
    y = _bf16_to_f64(st)
    unit = P.astype(np.float64) / np.maximum(np.linalg.norm(P.astype(np.float64), axis=1, keepdims=True), 1e-300)
    assert (np.abs(y - unit) <= np.abs(unit) * 2.0 ** -8 + 1e-30).all()      # half an ulp of 8 significant bits
    assert not st[4].any()
    norms = np.linalg.norm(y, axis=1)
    assert (np.abs(np.delete(norms, 4) - 1.0) < 2.0 ** -8).all()
    # torch's own bfloat16 rounding of the same fp32 products gives the same bits
    inv = (1.0 / np.linalg.norm(P.astype(np.float64), axis=1)).astype(np.float32)
    inv[4] = 0.0
    ref = torch.from_numpy((P * inv[:, None]).astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (st == ref).mean() > 0.9999            # fp64 vs fp32 norm can move a product across a rounding boundary


def test_score_equals_matrix_product_of_the_stored_values():
    C, N, M, k = 3, 20, 7, 192
    eta = [1.0, 0.5, 0.25]
    tr = [oracle.less16_store(_rows(N, k, 10 + c)) for c in range(C)]
    va = [oracle.less16_store(_rows(M, k, 20 + c)) for c in range(C)]
    sc, full = oracle.less16_score(tr, va, eta, want_full=True)
    want = sum(e * _bf16_to_f64(t) @ _bf16_to_f64(v).T for e, t, v in zip(eta, tr, va))
    np.testing.assert_allclose(full, want, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(sc, full.max(1))


def test_close_to_the_unquantised_cosine_and_self_similarity():
    C, N, M, k = 2, 16, 16, 512
    eta = [1.0, 0.75]
    Pt = [_rows(N, k, 30 + c) for c in range(C)]
    Pv = [p.copy() for p in Pt]                      # validation = train: the diagonal is the self-similarity
    full16 = oracle.less16_score([oracle.less16_store(p) for p in Pt], [oracle.less16_store(p) for p in Pv], eta,
                                 want_full=True)[1]
    exact = oracle.less_cosine(Pt, Pv, eta)
    assert np.abs(full16 - exact).max() < sum(eta) * 2.0 ** -7
    assert np.abs(np.diag(full16) - sum(eta)).max() < sum(eta) * 2.0 ** -7


def test_table1_storage_of_the_16_bit_store():
    """Table 1: the 16-bit store of "approximately 270K" examples (Sec. 4.1), k = 8192, four checkpoints,
    is listed as 16.54 GB: two bytes per stored value, as oracle.less16_store produces."""
    import os
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "table1_storage.txt"))
            if l.strip() and not l.startswith("#")]
    gb16 = float(dict(rows)["16"])
    bytes_per_example = oracle.less16_store(np.ones((1, 8192), dtype=np.float32)).nbytes * 4
    implied_examples = gb16 * 2 ** 30 / bytes_per_example
    assert abs(implied_examples - 270e3) < 0.01 * 270e3
