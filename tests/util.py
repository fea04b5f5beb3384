"""Shared helpers for the tests: seeded problems built from `datagen` only."""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache

import numpy as np
import torch

import cpu_codebooks as codebooks
import datagen


@dataclass
class Problem:
    kind: str
    X: np.ndarray  # base [N x D] fp32
    Y: np.ndarray  # queries [nq x D] fp32
    C: np.ndarray  # [k x D]
    P: np.ndarray  # [m x 256 x D/m]
    n: int

    @property
    def k(self):
        return self.C.shape[0]

    @property
    def D(self):
        return self.C.shape[1]

    @property
    def m(self):
        return self.P.shape[0]


@lru_cache(maxsize=None)
def problem(kind="sift", N=4000, nq=50, k=32, n=4, m=8, G=16, D=None, iters=4, seed=1, ntrain=None) -> Problem:
    """A small seeded problem: mixture data, Lloyd-trained C and P (CPU)."""
    mix = datagen.Mixture(kind, G, seed=datagen.MASTER_SEED + seed, dim=D)
    X = mix.base(N)
    Y = mix.queries(nq)
    T = mix.train_sample(ntrain or max(4 * k, min(N, 20000)))
    Cb, P = codebooks.train(T, k, n, m, iters=iters, seed=datagen.MASTER_SEED + seed)
    return Problem(kind, X.numpy(), Y.numpy(), Cb.numpy(), P.numpy(), n)
