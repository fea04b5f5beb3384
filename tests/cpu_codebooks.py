"""Codebook training fixture of the CPU tests: plain torch, fp32.

Lloyd iterations for the first-level codebook C and for the m PQ sub-codebooks (256 codewords
each) on line-quantisation residuals of a training sample, as in the paper's Sec. 3.1 / Sec. 5
set-up.  The codebooks are *inputs* of the method (both the oracle and the GPU library receive
them as plain arrays), so their quality only moves recall and has no bearing on parity.  The
residual step restates Eq. 7-8 and Eq. 12 on its own; it lives with the tests, outside the input
generators that the oracle and the library share, and neither of them calls it.
"""
from __future__ import annotations

import torch

from datagen import MASTER_SEED, STREAM_KMEANS, _gen


def _assign(X, Cb, chunk=None):
    if chunk is None:
        chunk = max(1024, (1 << 28) // Cb.shape[0])
    cn = (Cb * Cb).sum(1)
    out = torch.empty(X.shape[0], dtype=torch.int64, device=X.device)
    for s in range(0, X.shape[0], chunk):
        xs = X[s : s + chunk]
        d = cn[None, :] - 2.0 * (xs @ Cb.T)
        out[s : s + chunk] = d.argmin(1)
    return out


def lloyd(X: torch.Tensor, k: int, iters: int = 10, seed: int = MASTER_SEED, stream: int = 0) -> torch.Tensor:
    """k-means: seeded random initial centroids, `iters` Lloyd iterations; an
    empty cluster keeps its previous centroid."""
    g = _gen("cpu", seed, STREAM_KMEANS, stream)
    nt = X.shape[0]
    if nt >= k:
        init = torch.randperm(nt, generator=g)[:k]
    else:
        init = torch.randint(0, nt, (k,), generator=g)
    Cb = X[init.to(X.device)].clone()
    if nt < k:  # fewer samples than centroids: jitter duplicates apart
        Cb += 1e-3 * torch.randn(Cb.shape, generator=g).to(X.device) * (X.std() + 1e-6)
    for _ in range(iters):
        a = _assign(X, Cb)
        sums = torch.zeros_like(Cb).index_add_(0, a, X)
        cnt = torch.zeros(k, device=X.device, dtype=X.dtype).index_add_(0, a, torch.ones_like(a, dtype=X.dtype))
        nz = cnt > 0
        Cb[nz] = sums[nz] / cnt[nz, None]
    return Cb.contiguous()


def knn_graph(Cb: torch.Tensor, n: int, chunk: int = 4096):
    """n nearest other centroids of each centroid (fp32; only used to form
    training residuals here, never handed to the oracle or the library)."""
    k = Cb.shape[0]
    cn = (Cb * Cb).sum(1)
    S = torch.empty(k, n, dtype=torch.int64, device=Cb.device)
    for s in range(0, k, chunk):
        d = cn[s : s + chunk, None] + cn[None, :] - 2.0 * (Cb[s : s + chunk] @ Cb.T)
        r = torch.arange(s, min(s + chunk, k), device=Cb.device)
        d[r - s, r] = float("inf")
        S[s : s + chunk] = d.topk(n, dim=1, largest=False).indices
    return S


def line_residuals(X, Cb, S, lo=-0.25, hi=0.5, chunk=1 << 14):
    """x - anchor for the training sample, anchor on the best of the n lines of
    x's cell with the parameter snapped to the 256-value grid."""
    step = (hi - lo) / 255.0
    R = torch.empty_like(X)
    for s in range(0, X.shape[0], chunk):
        x = X[s : s + chunk]
        i = _assign(x, Cb)
        ci = Cb[i]
        sj = Cb[S[i]]  # [b, n, D]
        e = sj - ci[:, None, :]
        c = (e * e).sum(2).clamp_min(1e-30)
        z = x - ci
        lam = (z[:, None, :] * e).sum(2) / c
        d2 = (z * z).sum(1, keepdim=True) - c * lam * lam
        j = d2.argmin(1)
        rows = torch.arange(x.shape[0], device=x.device)
        lj = (torch.round(lam[rows, j] / step) * step).clamp(lo, hi)
        R[s : s + chunk] = z - lj[:, None] * e[rows, j]
    return R


def train(Xtrain: torch.Tensor, k: int, n: int, m: int, iters: int = 10, seed: int = MASTER_SEED,
          pq_sample: int = 1 << 18):
    """Returns (C [k x D], P [m x 256 x D/m]) fp32 on Xtrain's device."""
    D = Xtrain.shape[1]
    assert D % m == 0
    Cb = lloyd(Xtrain, k, iters, seed, 0)
    S = knn_graph(Cb, n)
    R = line_residuals(Xtrain[:pq_sample], Cb, S)
    ds = D // m
    P = torch.stack([lloyd(R[:, p * ds : (p + 1) * ds].contiguous(), 256, iters, seed, 1 + p) for p in range(m)])
    return Cb, P.contiguous()
