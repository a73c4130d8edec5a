"""Pins for the oracle's random matrix R(seed, m, j)  (paper Sec. 2.2 / 2.4: a random Gaussian or
Rademacher map; the paper fixes no generator, so what can be pinned is what the mathematics
fixes: balance, independence across rows / columns / seeds, and the normal quantiles)."""
import numpy as np
import pytest
from scipy.stats import norm

import oracle


def _words(seed, rows, nw, salt=0):
    return np.array([[oracle.word(seed, m, w, salt) for w in range(nw)] for m in rows],
                    dtype=np.uint64)


def test_every_bit_position_is_balanced_and_used_once():
    W = _words(0, range(64), 256)
    bits = ((W[..., None] >> np.arange(32, dtype=np.uint64)) & 1).astype(np.float64)
    n = W.size
    frac = bits.reshape(-1, 32).mean(0)
    assert np.all(np.abs(frac - 0.5) < 5 * 0.5 / np.sqrt(n))
    # the 32 columns of one word read 32 distinct bits: flipping through them recovers the word
    for m in (0, 5):
        for w in (0, 7):
            h = oracle.word(0, m, w)
            seen = 0
            cols = [oracle.r_entry(0, oracle.RADEMACHER, m, 32 * w + c) for c in range(32)]
            assert set(cols) <= {-1.0, 1.0}
            assert sum(1 for c in cols if c < 0) == bin(h).count("1")
            for c in range(32):
                b = 4 * (c % 8) + 3 - c // 8
                assert (cols[c] < 0) == bool((h >> b) & 1)
                seen |= 1 << b
            assert seen == 0xFFFFFFFF


def test_rows_columns_and_seeds_are_uncorrelated():
    d = 1 << 14
    R = np.array([[oracle.r_entry(3, 0, m, j) for j in range(0, d)] for m in range(24)])
    assert abs(R.mean()) < 5 / np.sqrt(R.size)
    Cr = (R @ R.T) / d
    off = Cr - np.eye(24)
    assert np.abs(off).max() < 5 / np.sqrt(d)
    # neighbouring columns (serial correlation inside and across words), lags 1..64
    for lag in (1, 2, 3, 4, 8, 31, 32, 33, 64):
        c = (R[:, :-lag] * R[:, lag:]).mean()
        assert abs(c) < 5 / np.sqrt(R[:, lag:].size)
    # another seed gives an unrelated matrix; the high half of the seed matters too
    for other in (4, 3 + (1 << 32)):
        R2 = np.array([[oracle.r_entry(other, 0, m, j) for j in range(0, 4096)] for m in range(8)])
        assert abs((R[:8, :4096] * R2).mean()) < 5 / np.sqrt(R2.size)


def test_avalanche_of_word_counter_and_row():
    # neighbouring counters / rows differ in about half of the 32 bits
    a = _words(9, [11], 2000)[0]
    flips = np.array([bin(int(x) ^ int(y)).count("1") for x, y in zip(a[:-1], a[1:])])
    assert abs(flips.mean() - 16) < 0.5
    b = np.array([oracle.word(9, m, 5) for m in range(2000)], dtype=np.uint64)
    flips = np.array([bin(int(x) ^ int(y)).count("1") for x, y in zip(b[:-1], b[1:])])
    assert abs(flips.mean() - 16) < 0.5
    assert len(set(int(x) for x in a)) > 1990 and len(set(int(x) for x in b)) > 1990


def test_rows_are_not_shifted_copies_of_each_other():
    # two row keys make word(m, w) = word(m', w + t) for all w practically impossible
    a = _words(1, range(32), 64)
    for t in range(1, 4):
        assert not np.any(np.all(a[:, t:][:, None, :] == a[:, :-t][None, :, :], axis=-1))


def test_gaussian_table_is_the_bf16_rounded_normal_quantiles():
    import torch
    T = oracle.gauss_table()
    ref = norm.ppf((np.arange(256) + 0.5) / 256.0)
    ref_bf16 = torch.tensor(ref, dtype=torch.float64).to(torch.float32).to(torch.bfloat16)
    np.testing.assert_array_equal(T, ref_bf16.to(torch.float64).numpy())
    np.testing.assert_array_equal(T, -T[::-1])
    assert abs(T.mean()) < 1e-12 and 0.97 < T.var() < 1.0
    assert np.all(np.diff(T) >= 0)


def test_gaussian_entries_follow_the_table_uniformly():
    T = oracle.gauss_table()
    vals = np.array([[oracle.r_entry(2, oracle.GAUSSIAN, m, j) for j in range(4096)]
                     for m in range(16)])
    assert set(np.unique(vals)) <= set(T)
    assert abs(vals.mean()) < 5 / np.sqrt(vals.size)
    assert abs(vals.var() - T.var()) < 0.03
    # bytes of one word feed four consecutive columns
    h = oracle.word(2, 3, 10, 1)
    for c in range(4):
        assert oracle.r_entry(2, oracle.GAUSSIAN, 3, 40 + c) == T[(h >> (8 * c)) & 0xFF]
    k = ((vals - vals.mean()) ** 4).mean() / vals.var() ** 2
    assert 2.6 < k < 3.1


def test_golden_words_file_matches():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "generator_words.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 16
    for seed, m, w, salt, hexword in rows:
        assert oracle.word(int(seed), int(m), int(w), int(salt)) == int(hexword, 16)
