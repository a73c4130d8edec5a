"""Pins of the oracle's aggregation over groups of validation examples (Sec. 4.1: selection by
"cumulative influence scores"; the paper gives no formula, so these pin the stated definitions:
group maximum, and fp32 mean in column order).  CPU only."""
import numpy as np
import pytest

import oracle


def _brute(full, ends, mode):
    N = full.shape[0]
    out = np.zeros((N, len(ends)), dtype=np.float32)
    for z in range(N):
        g0 = 0
        for t, g1 in enumerate(ends):
            vals = [np.float32(x) for x in full[z, g0:g1]]
            if mode == 0:
                out[z, t] = max(vals)
            else:
                s = np.float32(0.0)
                for v in vals:                      # one fp32 rounding per addition, column order
                    s = np.float32(s + v)
                out[z, t] = np.float32(s / np.float32(len(vals)))
            g0 = g1
    return out


@pytest.mark.parametrize("mode", [0, 1])
def test_aggregate_matches_brute_force(mode):
    rng = np.random.default_rng(5 + mode)
    full = (rng.standard_normal((37, 29)) * 10 ** rng.uniform(-3, 3, size=(37, 1))).astype(np.float32)
    ends = [1, 2, 9, 20, 29]
    got = oracle.aggregate(full, ends, mode)
    np.testing.assert_array_equal(got.view(np.uint32), _brute(full, ends, mode).view(np.uint32))


def test_one_group_maximum_is_the_score_of_the_north_star():
    """A single group over all validation examples reproduces oracle.score's max over val."""
    rng = np.random.default_rng(11)
    k, bits, C = 128, 4, 2
    t = [oracle.quantize(rng.standard_normal((50, k)).astype(np.float32), bits) for _ in range(C)]
    v = [oracle.quantize(rng.standard_normal((7, k)).astype(np.float32), bits) for _ in range(C)]
    sc, full = oracle.score([o[0] for o in t], [o[2] for o in t], [o[0] for o in v], [o[2] for o in v],
                            [1.0, 0.5], k, bits, want_full=True)
    np.testing.assert_array_equal(oracle.aggregate(full, [7], 0)[:, 0].view(np.uint32), sc.view(np.uint32))


def test_mean_special_cases_and_bounds():
    full = np.array([[1.0, 2.0, 3.0, 6.0], [-1.0, -1.0, -1.0, -1.0], [1e30, -1e30, 1.0, 1.0]], dtype=np.float32)
    m = oracle.aggregate(full, [4], 1)[:, 0]
    assert m[0] == np.float32(3.0) and m[1] == np.float32(-1.0)
    assert m[2] == np.float32(0.5)                   # ((1e30 - 1e30) + 1) + 1 = 2, in column order
    per = oracle.aggregate(full, [1, 2, 3, 4], 1)    # groups of one: the entries themselves
    np.testing.assert_array_equal(per, full)
    mx, mean = oracle.aggregate(full, [2, 4], 0), oracle.aggregate(full, [2, 4], 1)
    assert np.all(mean <= mx)                        # a mean never exceeds the maximum of its group
    # permuting the columns inside a group leaves its maximum unchanged
    np.testing.assert_array_equal(oracle.aggregate(full[:, [1, 0, 3, 2]], [2, 4], 0), mx)


def test_aggregate_rejects_bad_groups():
    full = np.zeros((2, 5), dtype=np.float32)
    for ends in ([5, 5], [3], [0, 5], [4, 3, 5], [6]):
        with pytest.raises(Exception):
            oracle.aggregate(full, ends, 0)
    with pytest.raises(Exception):
        oracle.aggregate(full, [5], 2)
