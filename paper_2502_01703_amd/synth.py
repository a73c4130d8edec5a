"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the HIP path and the CPU oracle (tests and the benchmark hand the same
tensors to each side).  It holds none of the method's arithmetic: no projection, no quantiser,
no scoring -- only random gradient-like vectors, planted correlated pairs and learning rates.

The paper measures on about 270K instruction-tuning examples with few-shot validation examples
(Sec. 4.1); those datasets are not available here, so these generators stand in for their
shapes, sizes and value distributions only.
"""
import math

import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def lognormal_scales(n, seed, device="cpu"):
    """Per-vector scale factors exp(N(0,1)): examples differ widely in gradient norm."""
    return torch.exp(torch.randn(n, generator=_gen(seed, device), device=device))


def gaussian_gradients(n, d, seed, device="cpu", dtype=torch.float32):
    """n vectors of N(0,1) entries, each multiplied by its own lognormal(0,1) scale."""
    g = _gen(seed, device)
    x = torch.randn(n, d, generator=g, device=device)
    s = torch.exp(torch.randn(n, 1, generator=g, device=device))
    return (x * s).to(dtype), s.flatten()


def student_t_gradients(n, d, seed, device="cpu", dtype=torch.bfloat16, nu=4, chunk_rows=None,
                        out=None):
    """n vectors of Student-t(nu) entries times a per-vector lognormal(0,1) scale.

    Built row-chunk by row-chunk so that a [64, 2^27] tensor never needs fp32 temporaries of
    its full size.  `out` may be a preallocated [n, d] tensor of `dtype`."""
    g = _gen(seed, device)
    if out is None:
        out = torch.empty(n, d, device=device, dtype=dtype)
    s = torch.exp(torch.randn(n, generator=g, device=device))
    if chunk_rows is None:
        chunk_rows = max(1, min(n, (1 << 26) // max(d, 1)))
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        z = torch.randn(r1 - r0, d, generator=g, device=device)
        chi = torch.zeros_like(z)
        for _ in range(nu):
            r = torch.randn(r1 - r0, d, generator=g, device=device)
            chi.addcmul_(r, r)
        z.mul_(torch.rsqrt(chi / nu))
        z.mul_(s[r0:r1, None])
        out[r0:r1] = z.to(dtype)
    return out, s


def planted_validation(train, scales, M, n_planted, seed, mix=0.5):
    """Validation vectors: the first n_planted are mix * x_p + scale_p * N(0,1) for distinct
    planted train rows p (true cosine = mix / sqrt(mix^2 + 1) for unit-variance rows); the rest
    are independent vectors of the same family.  Returns (val, planted_train_indices)."""
    device = train.device
    g = _gen(seed, device)
    N, d = train.shape
    perm = torch.randperm(N, generator=g, device=device)[:n_planted]
    val = torch.randn(M, d, generator=g, device=device)
    vs = torch.exp(torch.randn(M, generator=g, device=device))
    val[n_planted:] *= vs[n_planted:, None]
    val[:n_planted] = mix * train[perm].float() + scales[perm, None] * val[:n_planted]
    return val.to(train.dtype), perm


def config1(seed=1234, N=1024, M=64, d=16384, n_planted=32, device="cpu"):
    """Tiny CPU-checkable case: fp32 gradients, 32 planted pairs."""
    train, s = gaussian_gradients(N, d, seed, device=device, dtype=torch.float32)
    val, planted = planted_validation(train, s, M, n_planted, seed + 1)
    return train, val, planted


def projected_datastore(N, M, k, C, seed, planted_frac=0.02, rho=0.5, device="cpu"):
    """Pre-projected k-dim vectors for scoring-only runs: N(0,1) entries per checkpoint; a
    planted_frac share of the train rows is built to have cosine rho with one validation row
    each (train_p = rho * val_v + sqrt(1-rho^2) * noise, per checkpoint).
    Returns (train [C][N,k] fp32, val [C][M,k] fp32, planted_rows, planted_val)."""
    g = _gen(seed, device)
    n_pl = int(planted_frac * N)
    rows = torch.randperm(N, generator=g, device=device)[:n_pl]
    tgt = torch.randint(0, M, (n_pl,), generator=g, device=device)
    train, val = [], []
    for _ in range(C):
        v = torch.randn(M, k, generator=g, device=device)
        t = torch.randn(N, k, generator=g, device=device)
        if n_pl:
            t[rows] = rho * v[tgt] + math.sqrt(1.0 - rho * rho) * t[rows]
        train.append(t)
        val.append(v)
    return train, val, rows, tgt


def learning_rates(C):
    """Linearly decaying learning-rate weights, one per checkpoint: 1, 1-1/C, ..."""
    return [1.0 - i / C for i in range(C)]
