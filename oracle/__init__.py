"""Python face of the C oracle (ctypes, host memory only).

TEST INFRASTRUCTURE: imported only by tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg.  It never imports the HIP package and shares nothing with it.

Arrays are numpy; bfloat16 gradients are passed as uint16 bit patterns (dtype_code 1), which
is how `as_host_gradient` converts a torch.bfloat16 CPU tensor.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

F32, BF16 = 0, 1
RADEMACHER, GAUSSIAN = 0, 1

_c = ctypes
_i64, _i32, _u64, _u32 = _c.c_int64, _c.c_int32, _c.c_uint64, _c.c_uint32
_vp = _c.c_void_p


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build(verbose=False)
        L = _c.CDLL(_LIB_PATH)
        L.oracle_word.restype = _u32
        L.oracle_word.argtypes = [_u64, _u32, _u32, _u32]
        L.oracle_r_entry.restype = _c.c_double
        L.oracle_r_entry.argtypes = [_u64, _c.c_int, _u32, _u64]
        L.oracle_gauss_table.restype = None
        L.oracle_gauss_table.argtypes = [_vp]
        L.oracle_project_rows.restype = _c.c_int
        L.oracle_project_rows.argtypes = [_vp, _c.c_int, _i64, _i64, _i64, _i64, _c.c_int, _u64,
                                          _vp, _i32, _vp]
        L.oracle_project.restype = _c.c_int
        L.oracle_project.argtypes = [_vp, _c.c_int, _i64, _i64, _i64, _i64, _i32, _c.c_int, _u64,
                                     _c.c_int, _vp, _i64]
        L.oracle_code_bytes.restype = _i64
        L.oracle_code_bytes.argtypes = [_i32, _c.c_int]
        L.oracle_unpack.restype = _c.c_int
        L.oracle_unpack.argtypes = [_vp, _i64, _i32, _c.c_int, _vp]
        L.oracle_pack.restype = _c.c_int
        L.oracle_pack.argtypes = [_vp, _i64, _i32, _c.c_int, _vp]
        L.oracle_quantize_unpacked.restype = _c.c_int
        L.oracle_quantize_unpacked.argtypes = [_vp, _i64, _i64, _i32, _c.c_int, _c.c_int, _vp, _vp]
        L.oracle_quantize.restype = _c.c_int
        L.oracle_quantize.argtypes = [_vp, _i64, _i64, _i32, _c.c_int, _vp, _vp, _vp]
        L.oracle_quantize_absmean.restype = _c.c_int
        L.oracle_quantize_absmean.argtypes = [_vp, _i64, _i64, _i32, _c.c_int, _vp, _vp, _vp, _vp]
        L.oracle_score.restype = _c.c_int
        L.oracle_score.argtypes = [_vp, _vp, _vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _c.c_int,
                                   _vp, _vp]
        L.oracle_topk.restype = _c.c_int
        L.oracle_topk.argtypes = [_vp, _i64, _i64, _vp, _vp]
        L.oracle_aggregate.restype = _c.c_int
        L.oracle_aggregate.argtypes = [_vp, _i64, _c.c_int32, _vp, _c.c_int, _c.c_int, _vp]
        L.oracle_less_cosine.restype = _c.c_int
        L.oracle_less_cosine.argtypes = [_vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _vp]
        L.oracle_less16_store.restype = _c.c_int
        L.oracle_less16_store.argtypes = [_vp, _i64, _i64, _i32, _vp]
        L.oracle_less16_score.restype = _c.c_int
        L.oracle_less16_score.argtypes = [_vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _vp, _vp]
        L.oracle_score_mixed.restype = _c.c_int
        L.oracle_score_mixed.argtypes = [_vp, _vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _c.c_int, _vp, _vp]
        L.oracle_num_threads.restype = _c.c_int
        _lib = L
    return _lib


def _ptr(a):
    return _vp(a.ctypes.data)


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s: bad argument (rc=%d)" % (what, rc))


def as_host_gradient(G):
    """(array, dtype_code) for fp32 numpy/torch input or bfloat16 torch input (2-D, row-major)."""
    if isinstance(G, np.ndarray):
        if G.dtype == np.float32:
            return np.ascontiguousarray(G), F32
        if G.dtype == np.uint16:
            return np.ascontiguousarray(G), BF16
        raise TypeError("gradient must be float32 or uint16 (bfloat16 bits)")
    import torch
    G = G.detach().cpu().contiguous()
    if G.dtype == torch.float32:
        return G.numpy(), F32
    if G.dtype == torch.bfloat16:
        return G.view(torch.int16).numpy().view(np.uint16), BF16
    raise TypeError("gradient must be float32 or bfloat16")


def num_threads():
    return int(lib().oracle_num_threads())


def word(seed, m, w, salt=0):
    return int(lib().oracle_word(seed, m, w, salt))


def r_entry(seed, kind, m, j):
    return float(lib().oracle_r_entry(seed, kind, m, j))


def gauss_table():
    out = np.zeros(256, dtype=np.float64)
    lib().oracle_gauss_table(_ptr(out))
    return out


def project_rows(G, rows, kind=RADEMACHER, seed=0, d_offset=0):
    """Eq.(1) for the listed rows of R only; returns fp64 [n, len(rows)]."""
    A, dt = as_host_gradient(G)
    n, d = A.shape
    rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    out = np.zeros((n, rows.size), dtype=np.float64)
    _check(lib().oracle_project_rows(_ptr(A), dt, n, d, d, d_offset, kind, seed, _ptr(rows),
                                     rows.size, _ptr(out)), "project_rows")
    return out


def project(G, k, kind=RADEMACHER, seed=0, d_offset=0, P=None):
    """Eq.(1); returns fp32 [n, k].  With P given, accumulates into a copy of it."""
    A, dt = as_host_gradient(G)
    n, d = A.shape
    acc = 0
    if P is None:
        P = np.zeros((n, k), dtype=np.float32)
    else:
        P = np.array(P, dtype=np.float32, copy=True)
        acc = 1
    _check(lib().oracle_project(_ptr(A), dt, n, d, d, d_offset, k, kind, seed, acc, _ptr(P), k),
           "project")
    return P


def code_bytes(k, bits):
    return int(lib().oracle_code_bytes(k, bits))


def quantize(P, bits):
    """Eq.(4),(5) canonical; returns (codes uint8 [n, k*bits/8], S fp32 [n], rnorm fp32 [n])."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    n, k = P.shape
    codes = np.zeros((n, code_bytes(k, bits)), dtype=np.uint8)
    S = np.zeros(n, dtype=np.float32)
    rn = np.zeros(n, dtype=np.float32)
    _check(lib().oracle_quantize(_ptr(P), k, n, k, bits, _ptr(codes), _ptr(S), _ptr(rn)),
           "quantize")
    return codes, S, rn


def quantize_unpacked(P, bits, literal=False):
    """Integer codes int8 [n, k] and S; literal=True uses the real-number formula in fp64."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    n, k = P.shape
    q = np.zeros((n, k), dtype=np.int8)
    S = np.zeros(n, dtype=np.float32)
    _check(lib().oracle_quantize_unpacked(_ptr(P), k, n, k, bits, int(literal), _ptr(q), _ptr(S)),
           "quantize_unpacked")
    return q, S


def quantize_absmean(P, bits, want_unpacked=False):
    """Absmean variant (Sec. 5): (codes, S = mean|g|, rnorm[, q int8 [n, k]])."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    n, k = P.shape
    codes = np.zeros((n, code_bytes(k, bits)), dtype=np.uint8)
    q = np.zeros((n, k), dtype=np.int8) if want_unpacked else None
    S = np.zeros(n, dtype=np.float32)
    rn = np.zeros(n, dtype=np.float32)
    _check(lib().oracle_quantize_absmean(_ptr(P), k, n, k, bits, _ptr(codes),
                                         _ptr(q) if want_unpacked else None, _ptr(S), _ptr(rn)),
           "quantize_absmean")
    return (codes, S, rn, q) if want_unpacked else (codes, S, rn)


def unpack(codes, k, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    n = codes.shape[0]
    q = np.zeros((n, k), dtype=np.int8)
    _check(lib().oracle_unpack(_ptr(codes), n, k, bits, _ptr(q)), "unpack")
    return q


def pack(q, bits):
    q = np.ascontiguousarray(q, dtype=np.int8)
    n, k = q.shape
    codes = np.zeros((n, code_bytes(k, bits)), dtype=np.uint8)
    _check(lib().oracle_pack(_ptr(q), n, k, bits, _ptr(codes)), "pack")
    return codes


def _ptr_array(arrs):
    return (_vp * len(arrs))(*[a.ctypes.data for a in arrs])


def score(train_codes, train_rnorm, val_codes, val_rnorm, eta, k, bits, want_full=False):
    """Eq.(6),(7) + max over validation.  Lists of per-checkpoint arrays.
    Returns score fp32 [N] (and full fp32 [N, M] when want_full)."""
    C = len(train_codes)
    tc = [np.ascontiguousarray(a, dtype=np.uint8) for a in train_codes]
    vc = [np.ascontiguousarray(a, dtype=np.uint8) for a in val_codes]
    tr = [np.ascontiguousarray(a, dtype=np.float32) for a in train_rnorm]
    vr = [np.ascontiguousarray(a, dtype=np.float32) for a in val_rnorm]
    eta = np.ascontiguousarray(eta, dtype=np.float32)
    if not (len(tr) == len(vc) == len(vr) == eta.size == C):
        raise ValueError("oracle score: one entry per checkpoint is needed in every list")
    N, M = tc[0].shape[0], vc[0].shape[0]
    sc = np.zeros(N, dtype=np.float32)
    full = np.zeros((N, M), dtype=np.float32) if want_full else None
    _check(lib().oracle_score(_ptr_array(tc), _ptr_array(tr), _ptr_array(vc), _ptr_array(vr),
                              _ptr(eta), C, N, M, k, bits, _ptr(sc),
                              _ptr(full) if want_full else None), "score")
    return (sc, full) if want_full else sc


def topk(score_vec, k_sel):
    s = np.ascontiguousarray(score_vec, dtype=np.float32)
    idx = np.zeros(k_sel, dtype=np.int64)
    val = np.zeros(k_sel, dtype=np.float32)
    _check(lib().oracle_topk(_ptr(s), s.size, k_sel, _ptr(idx), _ptr(val)), "topk")
    return idx, val


def aggregate(full, group_end, mode):
    """Maximum (mode 0) or fp32 mean (mode 1) of full[N, M] over the column groups ending at group_end."""
    f = np.ascontiguousarray(full, dtype=np.float32)
    ge = np.ascontiguousarray(group_end, dtype=np.int32)
    out = np.zeros((f.shape[0], ge.size), dtype=np.float32)
    _check(lib().oracle_aggregate(_ptr(f), f.shape[0], f.shape[1], _ptr(ge), ge.size, mode, _ptr(out)), "aggregate")
    return out


def less_cosine(train_P, val_P, eta):
    """Eq.(2),(3): fp64 [N, M] LESS influence on un-quantised projections."""
    C = len(train_P)
    tp = [np.ascontiguousarray(a, dtype=np.float32) for a in train_P]
    vp = [np.ascontiguousarray(a, dtype=np.float32) for a in val_P]
    eta = np.ascontiguousarray(eta, dtype=np.float32)
    N, k = tp[0].shape
    M = vp[0].shape[0]
    out = np.zeros((N, M), dtype=np.float64)
    _check(lib().oracle_less_cosine(_ptr_array(tp), _ptr_array(vp), _ptr(eta), C, N, M, k,
                                    _ptr(out)), "less_cosine")
    return out


def less16_store(P):
    """LESS 16-bit datastore rows: bfloat16 bit patterns (uint16 [n, k]) of the normalised projections."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    n, k = P.shape
    out = np.zeros((n, k), dtype=np.uint16)
    _check(lib().oracle_less16_store(_ptr(P), k, n, k, _ptr(out)), "less16_store")
    return out


def less16_score(train16, val16, eta, want_full=False):
    """Eq.(2),(3) from stored bfloat16 rows, fp64: score [N] (and full [N, M])."""
    C = len(train16)
    tr = [np.ascontiguousarray(a, dtype=np.uint16) for a in train16]
    va = [np.ascontiguousarray(a, dtype=np.uint16) for a in val16]
    eta = np.ascontiguousarray(eta, dtype=np.float32)
    if not (len(va) == eta.size == C):
        raise ValueError("oracle less16_score: one entry per checkpoint is needed in every list")
    N, k = tr[0].shape
    M = va[0].shape[0]
    sc = np.zeros(N, dtype=np.float64)
    full = np.zeros((N, M), dtype=np.float64) if want_full else None
    _check(lib().oracle_less16_score(_ptr_array(tr), _ptr_array(va), _ptr(eta), C, N, M, k, _ptr(sc),
                                     _ptr(full) if want_full else None), "less16_score")
    return (sc, full) if want_full else sc


def score_mixed(train_codes, train_rnorm, val16, eta, k, bits, want_full=False):
    """b-bit train codes against stored bfloat16 validation rows (uint16 [M, k]), fp64: score [N] (and full [N, M])."""
    C = len(train_codes)
    tc = [np.ascontiguousarray(a, dtype=np.uint8) for a in train_codes]
    tr = [np.ascontiguousarray(a, dtype=np.float32) for a in train_rnorm]
    va = [np.ascontiguousarray(a, dtype=np.uint16) for a in val16]
    eta = np.ascontiguousarray(eta, dtype=np.float32)
    if not (len(tr) == len(va) == eta.size == C):
        raise ValueError("oracle score_mixed: one entry per checkpoint is needed in every list")
    N, M = tc[0].shape[0], va[0].shape[0]
    sc = np.zeros(N, dtype=np.float64)
    full = np.zeros((N, M), dtype=np.float64) if want_full else None
    _check(lib().oracle_score_mixed(_ptr_array(tc), _ptr_array(tr), _ptr_array(va), _ptr(eta), C, N, M, k, bits,
                                    _ptr(sc), _ptr(full) if want_full else None), "score_mixed")
    return (sc, full) if want_full else sc
