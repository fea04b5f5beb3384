"""Seeded synthetic inputs shared by the oracle tests and the GPU tests.

Nothing in this package implements the search method: it only makes inputs
(base vectors, queries) and, in ``datagen.codebooks``, trained codebooks that
both sides receive as plain arrays.  The generators are stand-ins for the
SIFT1B / DEEP1B collections used in the paper's Sec. 5 (same dimension, value
range and query-set size); no item of either collection is reproduced.

* SIFT-like: D = 128, G-component isotropic Gaussian mixture, component means
  uniform in [0, 128]^D, sigma 20, rounded and clipped to integers in [0, 255],
  stored as fp32.
* DEEP-like: D = 96, G-component mixture, means N(0, I), sigma 0.3, then
  L2-normalised.

Streams are independent functions of (master seed, stream, chunk): any chunk of
base vectors can be regenerated alone.  torch's CPU and GPU generators differ,
so a chunk is only reproducible on the device type it was first made on; tests
that need the same vectors on both sides generate once and copy.
"""
from __future__ import annotations

import torch

MASTER_SEED = 190100275
STREAM_MEANS, STREAM_BASE, STREAM_QUERY, STREAM_TRAIN, STREAM_KMEANS = 0, 1, 2, 3, 4
CHUNK = 1 << 20  # base vectors per independently seeded chunk


def _seed(seed: int, stream: int, chunk: int = 0) -> int:
    x = (seed * 0x9E3779B97F4A7C15 + stream * 0xBF58476D1CE4E5B9 + chunk * 0x94D049BB133111EB) & ((1 << 64) - 1)
    x ^= x >> 31
    x = (x * 0xD6E8FEB86659FD93) & ((1 << 64) - 1)
    x ^= x >> 29
    return x & ((1 << 62) - 1)


def _gen(device, seed, stream, chunk=0):
    g = torch.Generator(device=device)
    g.manual_seed(_seed(seed, stream, chunk))
    return g


class Mixture:
    """A seeded SIFT-like or DEEP-like Gaussian mixture."""

    def __init__(self, kind: str, components: int, seed: int = MASTER_SEED, dim: int | None = None):
        assert kind in ("sift", "deep")
        self.kind, self.G, self.seed = kind, int(components), int(seed)
        self.D = dim if dim is not None else (128 if kind == "sift" else 96)
        g = _gen("cpu", self.seed, STREAM_MEANS)
        if kind == "sift":
            self.means = torch.rand(self.G, self.D, generator=g) * 128.0
            self.sigma = 20.0
        else:
            self.means = torch.randn(self.G, self.D, generator=g)
            self.sigma = 0.3
        self._means_dev = {}

    def _means_on(self, device):
        key = str(device)
        if key not in self._means_dev:
            self._means_dev[key] = self.means.to(device)
        return self._means_dev[key]

    def _draw(self, count, gen, device):
        means = self._means_on(device)
        comp = torch.randint(0, self.G, (count,), generator=gen, device=device)
        x = torch.randn(count, self.D, generator=gen, device=device)
        x.mul_(self.sigma).add_(means[comp])
        if self.kind == "sift":
            x.round_().clamp_(0.0, 255.0)
        else:
            x.div_(x.norm(dim=1, keepdim=True).clamp_min_(1e-12))
        return x

    def base_chunk(self, chunk: int, device="cpu", count: int = CHUNK) -> torch.Tensor:
        """Base vectors chunk*CHUNK .. chunk*CHUNK+count-1 (count <= CHUNK)."""
        assert 0 < count <= CHUNK
        x = self._draw(CHUNK if count == CHUNK else count, _gen(device, self.seed, STREAM_BASE, chunk), device)
        return x

    def base(self, n: int, device="cpu") -> torch.Tensor:
        """The first n base vectors (ids 0..n-1)."""
        out, c = [], 0
        while n > 0:
            cnt = min(n, CHUNK)
            out.append(self.base_chunk(c, device, cnt))
            n -= cnt
            c += 1
        return out[0] if len(out) == 1 else torch.cat(out)

    def queries(self, nq: int, device="cpu") -> torch.Tensor:
        return self._draw(nq, _gen(device, self.seed, STREAM_QUERY), device)

    def train_sample(self, nt: int, device="cpu") -> torch.Tensor:
        """An independent sample of the same distribution for codebook training."""
        return self._draw(nt, _gen(device, self.seed, STREAM_TRAIN), device)


def exact_nn(base_chunks, Y: torch.Tensor, topk: int = 1):
    """Exact L2 nearest neighbours of Y among the concatenation of base_chunks
    (an iterable of [cnt x D] tensors on Y's device), as (dist, id).  Harness
    ground truth for Recall@K; fp32 GEMM form with fp64 norms."""
    nq = Y.shape[0]
    best_d = torch.full((nq, topk), float("inf"), device=Y.device, dtype=torch.float32)
    best_i = torch.full((nq, topk), -1, device=Y.device, dtype=torch.int64)
    yn = (Y.double() ** 2).sum(1)
    start = 0
    for X in base_chunks:
        for s in range(0, X.shape[0], 1 << 18):
            xs = X[s : s + (1 << 18)]
            d = (yn[:, None] + (xs.double() ** 2).sum(1)[None, :]).float() - 2.0 * (Y @ xs.T)
            dd, ii = torch.topk(d, min(topk, xs.shape[0]), dim=1, largest=False)
            cd = torch.cat([best_d, dd], 1)
            ci = torch.cat([best_i, ii + start + s], 1)
            best_d, sel = torch.topk(cd, topk, dim=1, largest=False)
            best_i = torch.gather(ci, 1, sel)
        start += X.shape[0]
    return best_d, best_i


def recall_at(found_ids: torch.Tensor, true_nn: torch.Tensor, K: int) -> float:
    """Recall@K of Sec. 5: fraction of queries whose true nearest neighbour is
    among the first K returned ids."""
    hit = (found_ids[:, :K].long() == true_nn.view(-1, 1).long()).any(1)
    return float(hit.float().mean())
