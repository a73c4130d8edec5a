"""qless_topk_noalloc (the entry point for callers that cannot allocate) against qless_topk: same
indices and the same score bits, on calls in a row that share the library's device array, the
later ones smaller than the first."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_01703_amd import binding as Q

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print("[case] " + msg, flush=True)


def _scores(N, seed, ties):
    rng = np.random.default_rng(seed)
    if ties:
        s = (rng.integers(-300, 300, size=N) / np.float32(256.0)).astype(np.float32)
        s[rng.integers(0, N, size=max(1, N // 40))] = np.float32(-0.0)
    else:
        s = rng.standard_normal(N).astype(np.float32)
    return torch.from_numpy(s).to(DEV)


def _compare(score, k_sel):
    ref_i, ref_v = Q.topk(score, k_sel)
    idx = torch.full((k_sel,), -1, dtype=torch.int64, device=DEV)
    val = torch.full((k_sel,), float("nan"), dtype=torch.float32, device=DEV)
    Q.topk_noalloc(score, idx, val)
    torch.cuda.synchronize()
    assert torch.equal(idx, ref_i)
    assert torch.equal(val.view(torch.int32), ref_v.view(torch.int32))


@pytest.mark.parametrize("ties", [False, True])
def test_noalloc_topk_matches_topk_on_calls_in_a_row(ties):
    # (N, k_sel): histogram launches + bitonic sort, then smaller: histogram launches + rank order,
    # then the single-workgroup selection, then the largest sizes accepted
    for step, (N, k_sel) in enumerate([(1300000, 40000), (270000, 13500), (20000, 1000), (1, 1),
                                       (Q.TOPK_NOALLOC_MAX_N, Q.TOPK_NOALLOC_MAX_SEL), (5000, 5000)]):
        _say("noalloc topk step %d: N=%d k_sel=%d ties=%s" % (step, N, k_sel, ties))
        _compare(_scores(N, 100 * step + int(ties), ties), k_sel)


def test_noalloc_topk_rejects_sizes_beyond_its_array():
    L = Q.lib()
    one = ctypes.c_void_p(16)        # never dereferenced: refused before anything is launched
    assert L.qless_topk_noalloc(one, Q.TOPK_NOALLOC_MAX_N + 1, 10, one, None, None) == 2
    assert L.qless_topk_noalloc(one, Q.TOPK_NOALLOC_MAX_N, Q.TOPK_NOALLOC_MAX_SEL + 1, one, None, None) == 2
    assert L.qless_topk_noalloc(one, 10, 11, one, None, None) == 1
    assert L.qless_topk_noalloc(None, 10, 5, one, None, None) == 1
    assert L.qless_topk_noalloc(one, 10, 0, None, None, None) == 0
