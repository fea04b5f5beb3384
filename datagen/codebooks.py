"""Seeded codebook training recipe run through the GPU library (inputs for the benchmark and the
full-size tests): seeded initial codebooks from the training sample, then every step by the
library's own calls.  This module holds no arithmetic of the method: it draws the initial rows and
sequences library calls; the library module is passed in by the caller.
"""
from __future__ import annotations

import torch

from . import MASTER_SEED, STREAM_KMEANS, _gen


def _seeded_init(X: torch.Tensor, k: int, seed: int, stream: int) -> torch.Tensor:
    """An initial codebook for Lloyd iterations: k seeded rows of X (jittered copies if X has fewer rows)."""
    g = _gen("cpu", seed, STREAM_KMEANS, stream)
    nt = X.shape[0]
    if nt >= k:
        init = torch.randperm(nt, generator=g)[:k]
    else:
        init = torch.randint(0, nt, (k,), generator=g)
    Cb = X[init.to(X.device)].clone()
    if nt < k:
        Cb += 1e-3 * torch.randn(Cb.shape, generator=g).to(X.device) * (X.std() + 1e-6)
    return Cb.contiguous()


def train_with_library(vlq, Xtrain: torch.Tensor, k: int, n: int, m: int, iters: int = 10, seed: int = MASTER_SEED,
                       pq_sample: int = 1 << 18, grid=(0.0, 0.0)):
    """Lloyd-trained C [k x D] and P [m x 256 x D/m], every step run by the GPU library: Lloyd iterations by
    vlq_kmeans, the n-NN graph by vlq_build_index, line-quantisation residuals by
    vlq_line_residuals, and one 256-word codebook per sub-space by vlq_kmeans again."""
    nt, D = Xtrain.shape
    assert D % m == 0
    ds = D // m
    Cb = _seeded_init(Xtrain, k, seed, 0)
    vlq.vlq_kmeans(Xtrain, nt, D, k, iters, Cb)
    # an index over the trained centroids (placeholder PQ codebooks) gives cells, lines and lambda bytes
    idx = vlq.vlq_build_index(vlq.vlq_params_t(D, k, n, m, grid[0], grid[1]), Cb, torch.zeros(m, 256, ds, device=Xtrain.device))
    try:
        ns = min(nt, pq_sample)
        R = torch.empty(ns, D, device=Xtrain.device)
        vlq.vlq_line_residuals(idx, Xtrain[:ns].contiguous(), ns, R)
    finally:
        vlq.vlq_index_free(idx)
    P = []
    for p in range(m):
        Rp = R[:, p * ds:(p + 1) * ds].contiguous()
        Pp = _seeded_init(Rp, 256, seed, 1 + p)
        vlq.vlq_kmeans(Rp, ns, ds, 256, iters, Pp)
        P.append(Pp)
    torch.cuda.synchronize()
    return Cb, torch.stack(P).contiguous()
