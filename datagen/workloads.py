"""The benchmark configurations (seeded synthetic stand-ins for SIFT1B / DEEP1B
at several scales) and the routine that materialises one of them on a GPU:
codebook training, streamed index build through the library's C ABI and exact
ground truth.  The library module is passed in by the caller, so this package
never imports the HIP path itself.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field

import torch

from . import CHUNK, MASTER_SEED, Mixture
from . import codebooks


@dataclass(frozen=True)
class Config:
    name: str
    kind: str  # "sift" (D = 128, integer valued) or "deep" (D = 96, unit norm)
    N: int
    G: int  # mixture components
    nq: int
    k: int  # first-level centroids
    n: int  # edges per centroid
    m: int  # code bytes
    w1: tuple  # probed cells (sweep); the last one is the headline operating point
    K: int = 100
    alpha: float = 0.25  # w2 = alpha * w1 * n (Sec. 3.3.1)
    w2_fixed: int = 0  # a stated number of sub-regions overrides alpha
    ntrain: int = 0
    batches: tuple = ()  # query batch sizes of the configuration's batch sweep
    Ks: tuple = ()  # result counts of the configuration's K sweep
    lam_lo: float = 0.0  # byte grid of lambda; (0, 0) = the library's default grid
    lam_hi: float = 0.0

    @property
    def D(self):
        return 128 if self.kind == "sift" else 96

    def w2(self, w1):
        return self.w2_fixed or max(1, int(self.alpha * w1 * self.n))


CONFIGS = {c.name: c for c in (
    Config("tiny_sift", "sift", 100_000, 64, 1_000, 256, 8, 8, (8,), w2_fixed=32, ntrain=20_000),
    Config("mid_sift", "sift", 10_000_000, 1_024, 10_000, 16_384, 32, 8, (8, 16, 32, 64), ntrain=1_000_000),
    Config("mid_deep", "deep", 100_000_000, 4_096, 10_000, 65_536, 32, 16, (16, 32, 64), ntrain=2_000_000),
    # the inverted-file baseline the paper compares against, expressed in this library's terms: four times the
    # centroids, one edge per cell and a lambda grid whose 256 values are all (numerically) zero, so every
    # anchor is the cell centroid, every probed cell is one list and the codes are residuals to the centroid
    Config("mid_sift_ivf", "sift", 10_000_000, 1_024, 10_000, 65_536, 1, 8, (8, 16, 32, 64, 128), alpha=1.0,
           ntrain=1_000_000, lam_lo=0.0, lam_hi=1e-20),
    Config("billion_sift", "sift", 1_000_000_000, 16_384, 10_000, 65_536, 32, 8, (16, 32, 64), ntrain=2_000_000),
    Config("billion_deep", "deep", 1_000_000_000, 16_384, 10_000, 65_536, 64, 16, (32, 64), ntrain=2_000_000,
           batches=(1, 16, 256, 10_000), Ks=(1, 10, 100)),
)}


@dataclass
class Workload:
    cfg: Config
    mix: Mixture
    C: torch.Tensor
    P: torch.Tensor
    Y: torch.Tensor
    idx: object  # library handle
    gt: torch.Tensor  # exact nearest neighbour id per query
    timings: dict = field(default_factory=dict)


def chunks(cfg: Config, n_points: int | None = None):
    n = cfg.N if n_points is None else n_points
    c = 0
    while n > 0:
        cnt = min(n, CHUNK)
        yield c, cnt
        n -= cnt
        c += 1


def materialise(vlq, cfg: Config, device="cuda:0", n_points: int | None = None, log=print, iters: int = 10,
                gt_rows: int | None = None) -> Workload:
    """Train codebooks, build the index chunk by chunk (vectors are generated,
    encoded, compared against the queries for ground truth, and dropped).
    gt_rows: exact nearest neighbours only for the first gt_rows queries (the rest get -1);
    the brute force over 10^9 points is the longest part of a build."""
    t0 = time.time()
    mix = Mixture(cfg.kind, cfg.G, seed=MASTER_SEED)
    T = mix.train_sample(cfg.ntrain, device)
    C, P = codebooks.train_with_library(vlq, T, cfg.k, cfg.n, cfg.m, iters=iters, seed=MASTER_SEED,
                                        grid=(cfg.lam_lo, cfg.lam_hi))
    del T
    torch.cuda.synchronize()
    t_train = time.time() - t0
    log(f"[{cfg.name}] codebooks trained in {t_train:.1f} s")
    Y = mix.queries(cfg.nq, device)
    prm = vlq.vlq_params_t(cfg.D, cfg.k, cfg.n, cfg.m, cfg.lam_lo, cfg.lam_hi)
    t0 = time.time()
    idx = vlq.vlq_build_index(prm, C, P)
    N = cfg.N if n_points is None else n_points
    vlq.vlq_index_reserve(idx, N)
    t_graph = time.time() - t0
    ng = cfg.nq if gt_rows is None else min(gt_rows, cfg.nq)
    best_d = torch.full((cfg.nq,), float("inf"), device=device)
    best_i = torch.full((cfg.nq,), -1, dtype=torch.int64, device=device)
    Yg = Y[:ng]
    yn = (Yg.double() ** 2).sum(1).float()
    t_add = t_gt = 0.0
    done = 0
    for c, cnt in chunks(cfg, N):
        X = mix.base_chunk(c, device, cnt)
        torch.cuda.synchronize()
        t1 = time.time()
        vlq.vlq_index_add(idx, X, cnt)
        torch.cuda.synchronize()
        t_add += time.time() - t1
        t1 = time.time()
        for s in range(0, cnt, 1 << 18):
            xs = X[s: s + (1 << 18)]
            d = (yn[:, None] + (xs * xs).sum(1)[None, :]) - 2.0 * (Yg @ xs.T)
            dd, ii = d.min(1)
            upd = dd < best_d[:ng]
            best_d[:ng] = torch.where(upd, dd, best_d[:ng])
            best_i[:ng] = torch.where(upd, ii + done + s, best_i[:ng])
        torch.cuda.synchronize()
        t_gt += time.time() - t1
        done += cnt
        del X
        if c % 16 == 15:
            log(f"[{cfg.name}] added {done} / {N} vectors ({t_add:.1f} s encode, {t_gt:.1f} s ground truth)")
    t1 = time.time()
    vlq.vlq_index_finalize(idx)
    torch.cuda.synchronize()
    t_fin = time.time() - t1
    log(f"[{cfg.name}] index built: {N} vectors, encode {t_add:.1f} s, finalize {t_fin:.1f} s")
    return Workload(cfg, mix, C, P, Y, idx, best_i,
                    dict(train_s=t_train, graph_s=t_graph, encode_s=t_add, ground_truth_s=t_gt, finalize_s=t_fin))


def visited_lists(vlq, idx, cfg: Config, sub: torch.Tensor):
    """The stored lists named in `sub` (any shape, labels i * n + j, -1 ignored), copied out of the
    library through vlq_index_get_lists and compacted: returns host arrays (off [k n + 1] int64 with
    zero length for every other list, ids, codes, lambda bytes) laid out like the library's own.
    Only marshalling: the oracle scans these lists on the host."""
    dev = sub.device
    nl = cfg.k * cfg.n
    N = vlq.vlq_index_ntotal(idx)
    off = torch.empty(nl + 1, dtype=torch.int64, device=dev)
    ids = torch.empty(N, dtype=torch.int32, device=dev)
    codes = torch.empty(N, cfg.m, dtype=torch.uint8, device=dev)
    lam = torch.empty(N, dtype=torch.uint8, device=dev)
    vlq.vlq_index_get_lists(idx, off, ids, codes, lam)
    torch.cuda.synchronize()
    labels = torch.unique(sub[sub >= 0].long())
    lens = off[labels + 1] - off[labels]
    total = int(lens.sum())
    first = torch.cumsum(lens, 0) - lens  # where each list starts in the compact arrays
    pos = torch.repeat_interleave(off[labels] - first, lens) + torch.arange(total, device=dev)
    off_c = torch.zeros(nl + 1, dtype=torch.int64, device=dev)
    off_c[labels + 1] = lens
    off_c = torch.cumsum(off_c, 0)
    out = (off_c.cpu().numpy(), ids[pos].cpu().numpy(), codes[pos].cpu().numpy(), lam[pos].cpu().numpy())
    del ids, codes, lam
    return out
