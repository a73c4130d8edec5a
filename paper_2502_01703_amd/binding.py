"""Thin ctypes binding over libqless.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/qless.h;
PyTorch supplies device memory and the current stream.  There is no CPU fallback: if the
library has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqless.so")
_lib = None

F32, BF16 = 0, 1
RADEMACHER, GAUSSIAN = 0, 1
MAX_CHECKPOINTS = 16
TOPK_NOALLOC_MAX_N, TOPK_NOALLOC_MAX_SEL = 4194304, 65536     # QLESS_TOPK_NOALLOC_MAX_* of qless.h

_c = ctypes
_i64, _i32, _u64, _u32, _vp, _sz = (_c.c_int64, _c.c_int32, _c.c_uint64, _c.c_uint32, _c.c_void_p,
                                    _c.c_size_t)

EXPORTS = {
    "qless_status_string": (_c.c_char_p, [_c.c_int]),
    "qless_init": (_c.c_int, []),
    "qless_project_workspace": (_sz, [_i64, _i64, _i32]),
    "qless_project": (_c.c_int, [_vp, _c.c_int, _i64, _i64, _i64, _i64, _i32, _c.c_int, _u64, _c.c_int,
                                 _vp, _i64, _vp, _sz, _vp]),
    "qless_generator_words": (_c.c_int, [_u64, _u32, _i32, _u32, _i32, _u32, _vp, _vp]),
    "qless_gaussian_table": (_c.c_int, [_vp]),
    "qless_quantize": (_c.c_int, [_vp, _i64, _i64, _i32, _c.c_int, _vp, _vp, _vp, _vp]),
    "qless_quantize_absmean": (_c.c_int, [_vp, _i64, _i64, _i32, _c.c_int, _vp, _vp, _vp, _vp]),
    "qless_project_quantize": (_c.c_int, [_vp, _c.c_int, _i64, _i64, _i64, _i64, _i32, _c.c_int, _u64, _c.c_int,
                                          _vp, _vp, _vp, _vp, _i64, _vp, _sz, _vp]),
    "qless_project_quantize_slice": (_c.c_int, [_vp, _c.c_int, _i64, _i64, _i64, _i64, _i32, _c.c_int, _u64, _c.c_int, _c.c_int,
                                                _vp, _i64, _vp, _i64, _c.c_int, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qless_score_workspace": (_sz, [_i64, _i32, _i32, _c.c_int, _c.c_int]),
    "qless_score": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _c.c_int, _vp, _vp,
                               _vp, _sz, _vp]),
    "qless_normalize16": (_c.c_int, [_vp, _i64, _i64, _i32, _vp, _vp]),
    "qless_score16_workspace": (_sz, [_i64, _i32, _i32, _c.c_int]),
    "qless_score16": (_c.c_int, [_vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "qless_score_mixed_workspace": (_sz, [_i64, _i32, _i32, _c.c_int, _c.c_int]),
    "qless_score_mixed": (_c.c_int, [_vp, _vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _c.c_int, _vp, _vp, _vp, _sz, _vp]),
    "qless_topk_workspace": (_sz, [_i64, _i64]),
    "qless_topk": (_c.c_int, [_vp, _i64, _i64, _vp, _vp, _vp, _sz, _vp]),
    "qless_topk_noalloc": (_c.c_int, [_vp, _i64, _i64, _vp, _vp, _vp]),
    "qless_aggregate": (_c.c_int, [_vp, _i64, _i32, _vp, _c.c_int, _c.c_int, _vp, _vp]),
    "qless_score_groups_workspace": (_sz, [_i64, _i32, _i32, _c.c_int, _c.c_int]),
    "qless_score_groups": (_c.c_int, [_vp, _vp, _vp, _vp, _vp, _c.c_int, _i64, _i32, _i32, _c.c_int, _vp, _c.c_int,
                                      _c.c_int, _vp, _vp, _sz, _vp]),
}


class QlessError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = lib().qless_status_string(status).decode()
        super().__init__("%s: %s (status %d)" % (what, msg, status))


def lib():
    """Loads libqless.so (built in-tree by `python -m paper_2502_01703_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libqless.so is not built: run `python -m paper_2502_01703_amd.build` "
                               "(there is no CPU fallback)")
        L = _c.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def init():
    """qless_init: one-time host-side set-up for the current device (needed before a graph capture)."""
    _check(lib().qless_init(), "qless_init")


def _stream():
    return _vp(torch.cuda.current_stream().cuda_stream)


def _check(status, what):
    if status != 0:
        raise QlessError(status, what)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("gradients must be float32 or bfloat16")


def _ws(nbytes, device, ws=None):
    if ws is not None:
        return ws
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def project_workspace(n, d_len, k):
    return int(lib().qless_project_workspace(n, d_len, k))


def project(G, k, kind=RADEMACHER, seed=0, d_offset=0, out=None, accumulate=False, ws=None):
    """qless_project: G [n, d] (device, fp32 or bf16, row stride free) -> P [n, k] fp32."""
    assert G.is_cuda and G.dim() == 2 and G.stride(1) == 1
    n, d = G.shape
    if out is None:
        assert not accumulate
        out = torch.empty(n, k, dtype=torch.float32, device=G.device)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1
    ldG = G.stride(0) if n > 1 else max(d, G.stride(0))
    w = _ws(project_workspace(n, d, k), G.device, ws)
    _check(lib().qless_project(_vp(G.data_ptr()), _dtype_code(G), n, d, ldG, d_offset, k, kind, seed,
                               int(accumulate), _vp(out.data_ptr()),
                               out.stride(0) if n > 1 else max(k, out.stride(0)),
                               _vp(w.data_ptr()), w.numel(), _stream()), "qless_project")
    return out


def generator_words(seed, m0, nrows, w0, nwords, salt=0, device="cuda"):
    out = torch.empty(nrows, nwords, dtype=torch.int32, device=device)
    _check(lib().qless_generator_words(seed, m0, nrows, w0, nwords, salt, _vp(out.data_ptr()), _stream()),
           "qless_generator_words")
    return out


def gaussian_table():
    buf = (_c.c_float * 256)()
    _check(lib().qless_gaussian_table(_c.cast(buf, _vp)), "qless_gaussian_table")
    return torch.tensor(list(buf), dtype=torch.float32)


def code_bytes(k, bits):
    return k * bits // 8


def quantize(P, bits, codes=None, S=None, rnorm=None, absmean=False):
    """qless_quantize (or qless_quantize_absmean): P [n, k] fp32 -> (codes uint8 [n, k*bits/8], S fp32 [n],
    rnorm fp32 [n])."""
    assert P.is_cuda and P.dtype == torch.float32 and P.dim() == 2 and P.stride(1) == 1
    n, k = P.shape
    dev = P.device
    if codes is None:
        codes = torch.empty(n, code_bytes(k, bits) if bits in (1, 2, 4, 8) else k, dtype=torch.uint8, device=dev)
    if S is None:
        S = torch.empty(n, dtype=torch.float32, device=dev)
    if rnorm is None:
        rnorm = torch.empty(n, dtype=torch.float32, device=dev)
    fn = lib().qless_quantize_absmean if absmean else lib().qless_quantize
    _check(fn(_vp(P.data_ptr()), P.stride(0) if n > 1 else max(k, P.stride(0)), n, k, bits,
              _vp(codes.data_ptr()), _vp(S.data_ptr()), _vp(rnorm.data_ptr()), _stream()),
           "qless_quantize_absmean" if absmean else "qless_quantize")
    return codes, S, rnorm


def project_quantize(G, k, bits, kind=RADEMACHER, seed=0, d_offset=0, want_P=False, ws=None):
    """qless_project_quantize: G [n, d] -> (codes, S, rnorm[, P]) in one call."""
    assert G.is_cuda and G.dim() == 2 and G.stride(1) == 1
    n, d = G.shape
    dev = G.device
    codes = torch.empty(n, code_bytes(k, bits) if bits in (1, 2, 4, 8) else k, dtype=torch.uint8, device=dev)
    S = torch.empty(n, dtype=torch.float32, device=dev)
    rnorm = torch.empty(n, dtype=torch.float32, device=dev)
    P = torch.empty(n, k, dtype=torch.float32, device=dev) if want_P else None
    ldG = G.stride(0) if n > 1 else max(d, G.stride(0))
    w = _ws(project_workspace(n, d, k), dev, ws)
    _check(lib().qless_project_quantize(_vp(G.data_ptr()), _dtype_code(G), n, d, ldG, d_offset, k, kind, seed,
                                        bits, _vp(codes.data_ptr()), _vp(S.data_ptr()), _vp(rnorm.data_ptr()),
                                        _vp(P.data_ptr()) if want_P else None, k,
                                        _vp(w.data_ptr()), w.numel(), _stream()), "qless_project_quantize")
    return (codes, S, rnorm, P) if want_P else (codes, S, rnorm)


def project_quantize_slice(G, k, d_offset, P, first, last, bits=1, kind=RADEMACHER, seed=0, P_other=None,
                           codes=None, S=None, rnorm=None, ws=None):
    """qless_project_quantize_slice: P (n x k fp32 accumulator) takes the slice G [n, d_len] at column d_offset of
    R; with last, P_other is added and the rows are quantised into codes, S, rnorm (returned)."""
    assert G.is_cuda and G.dim() == 2 and G.stride(1) == 1
    assert P.is_cuda and P.dtype == torch.float32 and P.stride(1) == 1 and P.shape[1] == k
    n, d = G.shape
    dev = G.device
    if last:
        if codes is None:
            codes = torch.empty(n, code_bytes(k, bits), dtype=torch.uint8, device=dev)
        if S is None:
            S = torch.empty(n, dtype=torch.float32, device=dev)
        if rnorm is None:
            rnorm = torch.empty(n, dtype=torch.float32, device=dev)
    ldG = G.stride(0) if n > 1 else max(d, G.stride(0))
    ldP = P.stride(0) if n > 1 else max(k, P.stride(0))
    ldO = 0 if P_other is None else (P_other.stride(0) if n > 1 else max(k, P_other.stride(0)))
    w = _ws(project_workspace(n, d, k), dev, ws)
    _check(lib().qless_project_quantize_slice(
        _vp(G.data_ptr()), _dtype_code(G), n, d, ldG, d_offset, k, kind, seed, int(first), int(last),
        _vp(P.data_ptr()), ldP, _vp(P_other.data_ptr()) if P_other is not None else None, ldO, bits,
        _vp(codes.data_ptr()) if last else None, _vp(S.data_ptr()) if last else None,
        _vp(rnorm.data_ptr()) if last else None, _vp(w.data_ptr()), w.numel(), _stream()),
        "qless_project_quantize_slice")
    return (codes, S, rnorm) if last else None


def score_workspace(N, M, k, bits, C):
    return int(lib().qless_score_workspace(N, M, k, bits, C))


def _ptr_array(tensors):
    return (_vp * len(tensors))(*[t.data_ptr() for t in tensors])


def score(train_codes, train_rnorm, val_codes, val_rnorm, eta, k, bits, want_score=True, want_full=False,
          score_out=None, full_out=None, ws=None):
    """qless_score: per-checkpoint lists of device tensors -> score [N] (and/or full [N, M])."""
    C = len(train_codes)
    assert len(train_rnorm) == C and len(val_codes) == C and len(val_rnorm) == C and len(eta) == C
    N, M = train_codes[0].shape[0], val_codes[0].shape[0]
    dev = val_codes[0].device
    for t in list(train_codes) + list(val_codes):
        assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()
    for t in list(train_rnorm) + list(val_rnorm):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    if want_score and score_out is None:
        score_out = torch.empty(N, dtype=torch.float32, device=dev)
    if want_full and full_out is None:
        full_out = torch.empty(N, M, dtype=torch.float32, device=dev)
    eta_arr = (_c.c_float * C)(*[float(e) for e in eta])
    w = _ws(score_workspace(N, M, k, bits, C), dev, ws)
    _check(lib().qless_score(_ptr_array(train_codes), _ptr_array(train_rnorm), _ptr_array(val_codes),
                             _ptr_array(val_rnorm), _c.cast(eta_arr, _vp), C, N, M, k, bits,
                             _vp(score_out.data_ptr()) if score_out is not None else None,
                             _vp(full_out.data_ptr()) if full_out is not None else None,
                             _vp(w.data_ptr()), w.numel(), _stream()), "qless_score")
    if want_score and want_full:
        return score_out, full_out
    return score_out if want_score else full_out


def normalize16(P, out=None):
    """qless_normalize16: P [n, k] fp32 -> unit rows in bfloat16 [n, k] (the 16-bit LESS store)."""
    assert P.is_cuda and P.dtype == torch.float32 and P.dim() == 2 and P.stride(1) == 1
    n, k = P.shape
    if out is None:
        out = torch.empty(n, k, dtype=torch.bfloat16, device=P.device)
    assert out.is_cuda and out.dtype == torch.bfloat16 and out.is_contiguous()
    _check(lib().qless_normalize16(_vp(P.data_ptr()), P.stride(0) if n > 1 else max(k, P.stride(0)), n, k,
                                   _vp(out.data_ptr()), _stream()), "qless_normalize16")
    return out


def score16_workspace(N, M, k, C):
    return int(lib().qless_score16_workspace(N, M, k, C))


def score16(train16, val16, eta, want_score=True, want_full=False, ws=None):
    """qless_score16: per-checkpoint lists of bfloat16 stores -> score [N] (and/or full [N, M])."""
    C = len(train16)
    assert len(val16) == C and len(eta) == C
    N, k = train16[0].shape
    M = val16[0].shape[0]
    dev = val16[0].device
    for t in list(train16) + list(val16):
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape[1] == k
    score_out = torch.empty(N, dtype=torch.float32, device=dev) if want_score else None
    full_out = torch.empty(N, M, dtype=torch.float32, device=dev) if want_full else None
    eta_arr = (_c.c_float * C)(*[float(e) for e in eta])
    w = _ws(score16_workspace(N, M, k, C), dev, ws)
    _check(lib().qless_score16(_ptr_array(train16), _ptr_array(val16), _c.cast(eta_arr, _vp), C, N, M, k,
                               _vp(score_out.data_ptr()) if want_score else None,
                               _vp(full_out.data_ptr()) if want_full else None,
                               _vp(w.data_ptr()), w.numel(), _stream()), "qless_score16")
    if want_score and want_full:
        return score_out, full_out
    return score_out if want_score else full_out


def score_mixed_workspace(N, M, k, bits, C):
    return int(lib().qless_score_mixed_workspace(N, M, k, bits, C))


def score_mixed(train_codes, train_rnorm, val16, eta, k, bits, want_score=True, want_full=False, ws=None):
    """qless_score_mixed: b-bit train codes against bfloat16 validation rows -> score [N] (and/or full [N, M])."""
    C = len(train_codes)
    assert len(train_rnorm) == C and len(val16) == C and len(eta) == C
    N, M = train_codes[0].shape[0], val16[0].shape[0]
    dev = val16[0].device
    for t in val16:
        assert t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.shape[1] == k
    for t in train_codes:
        assert t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous() and t.shape[1] == code_bytes(k, bits)
    score_out = torch.empty(N, dtype=torch.float32, device=dev) if want_score else None
    full_out = torch.empty(N, M, dtype=torch.float32, device=dev) if want_full else None
    eta_arr = (_c.c_float * C)(*[float(e) for e in eta])
    w = _ws(score_mixed_workspace(N, M, k, bits, C), dev, ws)
    _check(lib().qless_score_mixed(_ptr_array(train_codes), _ptr_array(train_rnorm), _ptr_array(val16),
                                   _c.cast(eta_arr, _vp), C, N, M, k, bits,
                                   _vp(score_out.data_ptr()) if want_score else None,
                                   _vp(full_out.data_ptr()) if want_full else None,
                                   _vp(w.data_ptr()), w.numel(), _stream()), "qless_score_mixed")
    if want_score and want_full:
        return score_out, full_out
    return score_out if want_score else full_out


def topk_workspace(N, k_sel):
    return int(lib().qless_topk_workspace(N, k_sel))


def topk(score_vec, k_sel, want_val=True, ws=None):
    """qless_topk: score [N] fp32 -> (idx int64 [k_sel], val fp32 [k_sel])."""
    assert score_vec.is_cuda and score_vec.dtype == torch.float32 and score_vec.is_contiguous()
    N = score_vec.numel()
    dev = score_vec.device
    idx = torch.empty(k_sel, dtype=torch.int64, device=dev)
    val = torch.empty(k_sel, dtype=torch.float32, device=dev) if want_val else None
    w = _ws(topk_workspace(N, k_sel), dev, ws)
    _check(lib().qless_topk(_vp(score_vec.data_ptr()), N, k_sel, _vp(idx.data_ptr()),
                            _vp(val.data_ptr()) if want_val else None, _vp(w.data_ptr()), w.numel(),
                            _stream()), "qless_topk")
    return (idx, val) if want_val else idx


def topk_noalloc(score_vec, idx, val=None):
    """qless_topk_noalloc: as topk, into the caller's idx (int64 [k_sel]) and val (fp32 [k_sel] or None);
    the call itself allocates nothing (the workspace is the library's own device array)."""
    assert score_vec.is_cuda and score_vec.dtype == torch.float32 and score_vec.is_contiguous()
    assert idx.is_cuda and idx.dtype == torch.int64 and idx.is_contiguous()
    assert val is None or (val.is_cuda and val.dtype == torch.float32 and val.numel() == idx.numel())
    _check(lib().qless_topk_noalloc(_vp(score_vec.data_ptr()), score_vec.numel(), idx.numel(),
                                    _vp(idx.data_ptr()), _vp(val.data_ptr()) if val is not None else None,
                                    _stream()), "qless_topk_noalloc")
    return idx, val


AGG_MAX, AGG_MEAN = 0, 1


def aggregate(full, group_end, mode=AGG_MAX, out=None):
    """qless_aggregate: full [N, M] fp32 -> [N, T] maximum or mean over the column groups ending at group_end."""
    assert full.is_cuda and full.dtype == torch.float32 and full.is_contiguous() and full.dim() == 2
    N, M = full.shape
    ge = (_c.c_int32 * len(group_end))(*[int(g) for g in group_end])
    if out is None:
        out = torch.empty(N, len(group_end), dtype=torch.float32, device=full.device)
    _check(lib().qless_aggregate(_vp(full.data_ptr()), N, M, _c.cast(ge, _vp), len(group_end), mode,
                                 _vp(out.data_ptr()), _stream()), "qless_aggregate")
    return out


def score_groups_workspace(N, M, k, bits, C):
    return int(lib().qless_score_groups_workspace(N, M, k, bits, C))


def score_groups(train_codes, train_rnorm, val_codes, val_rnorm, eta, k, bits, group_end, mode=AGG_MAX, out=None, ws=None):
    """qless_score_groups: influence aggregated over groups of validation columns -> [N, T]."""
    C = len(train_codes)
    assert len(train_rnorm) == C and len(val_codes) == C and len(val_rnorm) == C and len(eta) == C
    N, M = train_codes[0].shape[0], val_codes[0].shape[0]
    dev = val_codes[0].device
    T = len(group_end)
    ge = (_c.c_int32 * T)(*[int(g) for g in group_end])
    if out is None:
        out = torch.empty(N, T, dtype=torch.float32, device=dev)
    eta_arr = (_c.c_float * C)(*[float(e) for e in eta])
    w = _ws(score_groups_workspace(N, M, k, bits, C), dev, ws)
    _check(lib().qless_score_groups(_ptr_array(train_codes), _ptr_array(train_rnorm), _ptr_array(val_codes),
                                    _ptr_array(val_rnorm), _c.cast(eta_arr, _vp), C, N, M, k, bits,
                                    _c.cast(ge, _vp), T, mode, _vp(out.data_ptr()), _vp(w.data_ptr()), w.numel(),
                                    _stream()), "qless_score_groups")
    return out
