"""Codebook training pieces on the GPU against the oracle (through the C ABI): Lloyd iterations
(vlq_kmeans) and line-quantisation residuals (vlq_line_residuals), Sec. 2.1 / Sec. 3.2 / Sec. 5."""
import numpy as np
import pytest
import torch

from parity import GAP
from test_gpu_parity import DEV, dev, gpu_encode, make_index
from util import problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vlq():
    import paper_1901_00275_amd as vlq

    vlq.lib()
    return vlq


def _sample(nt, D, G, seed, integer=False):
    rng = np.random.default_rng(seed)
    means = rng.uniform(0, 100, size=(G, D))
    X = means[rng.integers(0, G, nt)] + rng.normal(scale=6.0, size=(nt, D))
    if integer:
        X = np.rint(X)
    return X.astype(np.float32), rng


def _kmeans(vlq, X, C0, iters, want_assign=True):
    nt, D = X.shape
    k = C0.shape[0]
    Cd = dev(C0.copy())
    a = torch.empty(nt, dtype=torch.int32, device=DEV) if want_assign else None
    c = torch.empty(k, dtype=torch.int32, device=DEV) if want_assign else None
    vlq.vlq_kmeans(dev(X), nt, D, k, iters, Cd, a, c)
    torch.cuda.synchronize()
    return Cd.cpu().numpy(), (a.cpu().numpy() if want_assign else None), (c.cpu().numpy() if want_assign else None)


def _check_assign(cell, o_cell, cd, what):
    diff = np.nonzero(cell != o_cell)[0]
    for t in diff:  # only inside the oracle's tie band
        assert cd[t, 1] - cd[t, 0] <= GAP * max(cd[t, 1], 1e-30), f"{what}: row {t} assigned to {cell[t]}, oracle {o_cell[t]}"
    return len(diff)


@pytest.mark.parametrize("nt,D,k,integer", [
    (20000, 32, 300, False),   # bf16 shortlist, several ragged tiles
    (9000, 128, 64, True),     # bf16 shortlist, integer-valued data (no low halves)
    (7000, 12, 40, False),     # fp32 shortlist
    (30000, 16, 256, False),   # the shape of a PQ sub-codebook
])
def test_lloyd_iterations_against_oracle(vlq, oracle_mod, nt, D, k, integer):
    X, rng = _sample(nt, D, 24, 11 + D, integer)
    C0 = X[rng.choice(nt, k, replace=False)].copy()
    C0[-1] = 1e4  # a centroid nobody is near: must stay where it is
    # assignment alone (iters = 0)
    Cs, a0, n0 = _kmeans(vlq, X, C0, 0)
    assert np.array_equal(Cs, C0)
    o_cell, cd = oracle_mod.vq_assign(C0, X)
    soft = _check_assign(a0, o_cell, cd, "iters=0")
    assert soft <= 3 and np.array_equal(n0, np.bincount(a0, minlength=k)) and n0[-1] == 0
    # three iterations, one at a time, each checked against the oracle's step from the same start
    Cc = C0
    for it in range(3):
        Cn, _, _ = _kmeans(vlq, X, Cc, 1, want_assign=False)
        Co, o_cell, cd = oracle_mod.lloyd_step(Cc, X)
        _, a_same, _ = _kmeans(vlq, X, Cc, 0)
        _check_assign(a_same, o_cell, cd, f"iteration {it}")
        agree = np.ones(k, bool)
        for t in np.nonzero(a_same != o_cell)[0]:
            agree[a_same[t]] = agree[o_cell[t]] = False
        scale = np.abs(X).max()
        assert np.allclose(Cn[agree], Co[agree], rtol=2e-7, atol=1e-6 * scale), f"iteration {it}"
        assert np.array_equal(Cn[-1], C0[-1])
        Cc = Cn
    # one call with three iterations is the same computation, bit for bit, and repeatable
    C3, a3, n3 = _kmeans(vlq, X, C0, 3)
    assert np.array_equal(C3, Cc)
    C3b, a3b, n3b = _kmeans(vlq, X, C0, 3)
    assert np.array_equal(C3, C3b) and np.array_equal(a3, a3b) and np.array_equal(n3, n3b)
    assert np.array_equal(n3, np.bincount(a3, minlength=k)) and n3.sum() == nt


def test_kmeans_rejects_bad_arguments(vlq):
    X = torch.zeros(10, 4, device=DEV)
    Cd = torch.zeros(2, 4, device=DEV)
    for args in [(None, 10, 4, 2, 1, Cd), (X, 0, 4, 2, 1, Cd), (X, 10, 0, 2, 1, Cd), (X, 10, 4, 0, 1, Cd),
                 (X, 10, 4, 2, -1, Cd), (X, 10, 4, 2, 1, None)]:
        with pytest.raises(vlq.VlqError):
            vlq.vlq_kmeans(*args)
    # all-zero data, more centroids than distinct points: nothing moves, nothing breaks
    vlq.vlq_kmeans(X, 10, 4, 2, 2, Cd)
    torch.cuda.synchronize()
    assert (Cd == 0).all()


@pytest.mark.parametrize("kind,D", [("sift", None), ("deep", None), ("sift", 12)])
def test_line_residuals_against_oracle(vlq, oracle_mod, kind, D):
    pr = problem(kind=kind, N=4000, k=64, n=6, m=4, G=16, nq=5, D=D)
    idx = make_index(vlq, pr)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        cell, edge, lamq, _ = gpu_encode(vlq, idx, pr.X, pr.m)
        R = torch.empty(len(pr.X), pr.D, device=DEV)
        vlq.vlq_line_residuals(idx, dev(pr.X), len(pr.X), R)
        torch.cuda.synchronize()
        Ro = oracle_mod.line_residual(pr.C, S, pr.X, cell, edge, lamq)  # for the GPU's own (validated) choices
        # formed in fp64, rounded once
        assert (np.abs(R.cpu().numpy() - Ro) <= 2.0 ** -23 * np.abs(Ro) + 1e-30).all()
    finally:
        vlq.vlq_index_free(idx)
