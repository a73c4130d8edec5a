"""Host-side checks of the HIP library that need no GPU: it loads, exports every symbol the
header declares, and refuses bad arguments before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_01703_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE = 0, 1, 2, 3


def test_header_symbols_are_all_exported():
    text = open(os.path.join(ROOT, "include", "qless.h")).read()
    declared = set(re.findall(r"\b(qless_[a-z0-9_]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    L = binding.lib()
    names = [L.qless_status_string(i).decode() for i in range(5)]
    assert names[0] == "ok" and len(set(names)) == 5


def test_project_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)       # never dereferenced: every call below must fail validation first
    f = L.qless_project
    assert f(one, 1, -1, 64, 64, 0, 64, 0, 0, 0, one, 64, one, 1 << 30, None) == INVALID
    assert f(one, 1, 4, 64, 32, 0, 64, 0, 0, 0, one, 64, one, 1 << 30, None) == INVALID      # ldG < d
    assert f(one, 1, 4, 64, 64, 0, 64, 0, 0, 0, one, 32, one, 1 << 30, None) == INVALID      # ldP < k
    assert f(None, 1, 4, 64, 64, 0, 64, 0, 0, 0, one, 64, one, 1 << 30, None) == INVALID
    assert f(one, 1, 4, 64, 64, 0, 100, 0, 0, 0, one, 100, one, 1 << 30, None) == UNSUPPORTED  # k % 64
    assert f(one, 1, 4, 64, 64, 8, 64, 0, 0, 0, one, 64, one, 1 << 30, None) == UNSUPPORTED    # offset % 32
    assert f(one, 7, 4, 64, 64, 0, 64, 0, 0, 0, one, 64, one, 1 << 30, None) == UNSUPPORTED    # dtype
    assert f(one, 1, 4, 64, 64, 0, 64, 5, 0, 0, one, 64, one, 1 << 30, None) == UNSUPPORTED    # kind
    need = L.qless_project_workspace(4, 64, 64)
    assert need == 4 * 64 * 4
    assert f(one, 1, 4, 64, 64, 0, 64, 0, 0, 0, one, 64, one, need - 1, None) == WORKSPACE
    assert f(one, 1, 4, 64, 64, 0, 64, 0, 0, 0, one, 64, None, 0, None) == WORKSPACE
    assert f(one, 1, 0, 64, 64, 0, 64, 0, 0, 0, None, 64, None, 0, None) == OK                # n = 0


def test_project_quantize_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)
    f = L.qless_project_quantize
    a = lambda G=one, n=4, d=64, ldG=64, off=0, k=64, bits=8, codes=one, P=None, ldP=0, ws=one, wsb=1 << 30: (
        G, 1, n, d, ldG, off, k, 0, 0, bits, codes, one, one, P, ldP, ws, wsb, None)
    assert f(*a(d=0)) == INVALID
    assert f(*a(codes=None)) == INVALID
    assert f(*a(G=None)) == INVALID
    assert f(*a(P=one, ldP=32)) == INVALID
    assert f(*a(bits=3)) == UNSUPPORTED
    assert f(*a(k=96)) == UNSUPPORTED
    assert f(*a(off=16)) == UNSUPPORTED
    assert f(*a(ws=None, wsb=0)) == WORKSPACE
    assert f(*a(ws=ctypes.c_void_p(8))) == WORKSPACE
    assert f(*a(wsb=64)) == WORKSPACE
    assert f(*a(n=0, codes=None)) == OK


def test_quantize_score_topk_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)
    q = L.qless_quantize
    assert q(one, 64, 4, 64, 3, one, one, one, None) == UNSUPPORTED
    assert q(one, 96, 4, 96, 8, one, one, one, None) == UNSUPPORTED
    assert q(one, 32, 4, 64, 8, one, one, one, None) == INVALID
    assert q(None, 64, 4, 64, 8, one, one, one, None) == INVALID
    assert q(None, 64, 0, 64, 8, None, None, None, None) == OK
    qm = L.qless_quantize_absmean
    assert qm(one, 64, 4, 64, 3, one, one, one, None) == UNSUPPORTED
    assert qm(one, 32, 4, 64, 8, one, one, one, None) == INVALID
    assert qm(one, 64, 4, 64, 8, None, one, one, None) == INVALID
    assert qm(None, 64, 0, 64, 8, None, None, None, None) == OK
    ptrs = (ctypes.c_void_p * 1)(16)
    eta = (ctypes.c_float * 1)(1.0)
    s = L.qless_score
    args = lambda C=1, N=4, M=2, k=64, bits=8, score=one, full=None: (
        ptrs, ptrs, ptrs, ptrs, ctypes.cast(eta, ctypes.c_void_p), C, N, M, k, bits, score, full, None, 0, None)
    assert s(*args(C=0)) == INVALID
    assert s(*args(C=17)) == UNSUPPORTED
    assert s(*args(M=0)) == INVALID
    assert s(*args(bits=3)) == UNSUPPORTED
    assert s(*args(k=100)) == UNSUPPORTED
    assert s(*args(score=None)) == INVALID
    assert s(*args(N=0)) == OK
    bad = (ctypes.c_void_p * 1)(8)           # codes must be 16-byte aligned
    assert s(bad, ptrs, ptrs, ptrs, ctypes.cast(eta, ctypes.c_void_p), 1, 4, 2, 64, 8, one, None, None, 0, None) == INVALID
    nz = L.qless_normalize16
    assert nz(one, 32, 4, 64, one, None) == INVALID
    assert nz(one, 96, 4, 96, one, None) == UNSUPPORTED
    assert nz(None, 64, 0, 64, None, None) == OK
    s16 = L.qless_score16
    a16 = lambda C=1, N=4, M=2, k=64, score=one, p=ptrs: (p, p, ctypes.cast(eta, ctypes.c_void_p), C, N, M, k,
                                                         score, None, None, 0, None)
    assert s16(*a16(C=0)) == INVALID
    assert s16(*a16(k=96)) == UNSUPPORTED
    assert s16(*a16(k=65536)) == UNSUPPORTED
    assert s16(*a16(score=None)) == INVALID
    assert s16(*a16(p=bad)) == INVALID
    assert s16(*a16()) == WORKSPACE
    assert s16(*a16(N=0)) == OK
    assert L.qless_score16_workspace(1000, 100, 512, 2) >= 2 * 128 * 1024
    t = L.qless_topk
    assert t(one, 10, 11, one, None, one, 1 << 20, None) == INVALID
    assert t(one, 10, -1, one, None, one, 1 << 20, None) == INVALID
    assert t(one, 10, 5, one, None, one, 8, None) == WORKSPACE
    assert t(one, 10, 0, None, None, None, 0, None) == OK
    assert L.qless_topk_workspace(270000, 13500) >= 16384 * 8 + 256 * 4      # selected keys (padded) + histogram
    ag = L.qless_aggregate
    ends = lambda *e: ctypes.cast((ctypes.c_int32 * len(e))(*e), ctypes.c_void_p)
    assert ag(one, 0, 5, ends(2, 5), 2, 0, one, None) == OK
    assert ag(one, 0, 5, ends(2, 4), 2, 0, one, None) == INVALID               # last end != M
    assert ag(one, 0, 5, ends(3, 3, 5), 3, 1, one, None) == INVALID            # empty group
    assert ag(one, 0, 5, ends(5), 1, 2, one, None) == UNSUPPORTED              # unknown mode
    assert ag(one, 0, 5, None, 1, 0, one, None) == INVALID
    assert ag(one, 0, 100, ends(*range(1, 66)), 65, 0, one, None) == UNSUPPORTED   # more than QLESS_MAX_GROUPS


def _golden_gaussian_table():
    path = os.path.join(ROOT, "tests", "golden", "gaussian_table_bf16.txt")
    bits = np.array([int(l, 16) for l in open(path) if not l.startswith("#")], dtype=np.uint32)
    assert bits.size == 256
    return (bits << 16).view(np.float32).astype(np.float64)


def test_gaussian_table_matches_the_stored_table_and_the_oracle():
    """The library's table is a constant array; the oracle computes its own with the host's math library; both
    must equal the stored bfloat16 bit patterns (a different libm must not move an entry)."""
    import oracle
    gold = _golden_gaussian_table()
    np.testing.assert_array_equal(binding.gaussian_table().numpy().astype(np.float64), gold)
    np.testing.assert_array_equal(oracle.gauss_table(), gold)
    np.testing.assert_array_equal(gold, -gold[::-1])


def test_gaussian_columns_end_at_2_to_34_on_both_sides():
    """The Gaussian stream numbers words of four columns with 32 bits: a column range past 2^34 is refused by
    the library (before any launch) and by the oracle; the Rademacher family goes on to 2^36."""
    import oracle
    L = binding.lib()
    one = ctypes.c_void_p(16)
    f = L.qless_project
    off = (1 << 34) - 64
    need = L.qless_project_workspace(4, 128, 64)
    assert f(one, 1, 4, 128, 128, off, 64, 1, 0, 0, one, 64, one, need, None) == UNSUPPORTED       # Gaussian, ends past 2^34
    assert f(one, 1, 0, 128, 128, off, 64, 0, 0, 0, one, 64, one, need, None) == OK                # Rademacher (n = 0: no launch)
    assert f(one, 1, 0, 64, 64, off, 64, 1, 0, 0, one, 64, one, need, None) == OK                  # Gaussian, ends at 2^34
    G = np.zeros((1, 128), dtype=np.float32)
    with pytest.raises(Exception):
        oracle.project_rows(G, [0], kind=oracle.GAUSSIAN, d_offset=off)
    assert oracle.project_rows(G[:, :64], [0], kind=oracle.GAUSSIAN, d_offset=off).shape == (1, 1)
    assert oracle.project_rows(G, [0], kind=oracle.RADEMACHER, d_offset=off).shape == (1, 1)


def test_misaligned_workspaces_and_codes_are_refused():
    L = binding.lib()
    one, odd = ctypes.c_void_p(16), ctypes.c_void_p(18)
    assert L.qless_topk(one, 10, 5, one, None, odd, 1 << 30, None) == WORKSPACE
    need = L.qless_project_workspace(4, 64, 64)
    assert L.qless_project(one, 1, 4, 64, 64, 0, 64, 0, 0, 0, one, 64, odd, need + 64, None) == WORKSPACE
    assert L.qless_quantize(one, 64, 4, 64, 8, odd, one, one, None) == INVALID
    assert L.qless_quantize_absmean(one, 64, 4, 64, 8, odd, one, one, None) == INVALID


def test_score_mixed_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)
    ptrs = (ctypes.c_void_p * 1)(16)
    eta = (ctypes.c_float * 1)(1.0)
    f = L.qless_score_mixed
    a = lambda C=1, N=4, M=2, k=64, bits=8, score=one, ws=one, wsb=1 << 30, tc=ptrs: (
        tc, ptrs, ptrs, ctypes.cast(eta, ctypes.c_void_p), C, N, M, k, bits, score, None, ws, wsb, None)
    assert f(*a(C=0)) == INVALID
    assert f(*a(M=0)) == INVALID
    assert f(*a(score=None)) == INVALID
    assert f(*a(bits=3)) == UNSUPPORTED
    assert f(*a(k=100)) == UNSUPPORTED
    assert f(*a(k=65536)) == UNSUPPORTED
    assert f(*a(ws=None)) == WORKSPACE
    assert f(*a(wsb=16)) == WORKSPACE
    assert f(*a(ws=ctypes.c_void_p(24))) == WORKSPACE
    assert f(*a(N=0, ws=None, wsb=0)) == OK
    need = L.qless_score_mixed_workspace(20000, 100, 1024, 4, 2)
    assert need >= 2 * 8192 * 1024 * 2
    assert L.qless_score_mixed_workspace(4, 2, 64, 3, 1) == 0


def test_project_quantize_slice_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)
    f = L.qless_project_quantize_slice
    a = lambda n=4, d=64, k=64, first=1, last=1, P=one, ldP=64, other=None, ldO=0, bits=8, codes=one, ws=one, wsb=1 << 30, off=0: (
        one, 1, n, d, 64, off, k, 0, 0, first, last, P, ldP, other, ldO, bits, codes, one, one, ws, wsb, None)
    assert f(*a(P=None)) == INVALID
    assert f(*a(ldP=32)) == INVALID
    assert f(*a(other=one, ldO=32)) == INVALID
    assert f(*a(last=0, other=one, ldO=64)) == INVALID          # a second accumulator is joined on the last slice only
    assert f(*a(codes=None)) == INVALID
    assert f(*a(codes=ctypes.c_void_p(18))) == INVALID
    assert f(*a(bits=5)) == UNSUPPORTED
    assert f(*a(off=8)) == UNSUPPORTED
    assert f(*a(ws=None, wsb=0)) == WORKSPACE
    assert f(*a(n=0, P=None, codes=None, ws=None, wsb=0)) == OK


def test_score_groups_argument_validation():
    L = binding.lib()
    one = ctypes.c_void_p(16)
    ptrs = (ctypes.c_void_p * 1)(16)
    eta = (ctypes.c_float * 1)(1.0)
    ends = lambda *v: (ctypes.c_int32 * len(v))(*v)
    f = L.qless_score_groups
    a = lambda N=4, M=5, k=64, bits=8, ge=ends(2, 5), T=2, mode=0, out=one, ws=one, wsb=1 << 30: (
        ptrs, ptrs, ptrs, ptrs, ctypes.cast(eta, ctypes.c_void_p), 1, N, M, k, bits, ge, T, mode, out, ws, wsb, None)
    assert f(*a(ge=ends(2, 4))) == INVALID                 # last end != M
    assert f(*a(ge=ends(3, 3, 5), T=3)) == INVALID         # empty group
    assert f(*a(ge=None)) == INVALID
    assert f(*a(mode=2)) == UNSUPPORTED
    assert f(*a(bits=3)) == UNSUPPORTED
    assert f(*a(out=None)) == INVALID
    assert f(*a(ws=None)) == WORKSPACE
    assert f(*a(wsb=8)) == WORKSPACE
    assert f(*a(N=0, out=None, ws=None, wsb=0)) == OK
    assert L.qless_score_groups_workspace(1000, 300, 1024, 1, 4) == L.qless_score_groups_workspace(1000, 300, 1024, 1, 4) > 0
