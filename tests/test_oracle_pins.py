"""Pins of the CPU oracle against things other than itself: hand-worked values,
closed forms, library routines (scipy cdist, numpy lstsq), brute-force
enumeration and special cases that reduce to textbook methods."""
import os

import numpy as np
import pytest
from scipy.spatial.distance import cdist

from util import problem

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].replace("|", " ").split()
        if line:
            out.append([float(v) for v in line])
    return np.array(out)


# ---- Eq. 7 / Eq. 8 / Eq. 9 ------------------------------------------------


def test_line_examples_by_hand(oracle_mod):
    for r in _rows("line_quantization_examples.txt"):
        ci, cj, x = r[0:2], r[2:4], r[4:6]
        a, b, c, lam, d2 = r[6:11]
        anchor = r[11:13]
        # the fixture itself is consistent with plain geometry
        assert np.isclose(((x - ci) ** 2).sum(), a) and np.isclose(((x - cj) ** 2).sum(), b)
        assert np.isclose(((ci - cj) ** 2).sum(), c)
        assert np.allclose((1 - lam) * ci + lam * cj, anchor)
        assert np.isclose(((x - anchor) ** 2).sum(), d2)
        # the oracle reproduces it
        assert oracle_mod.line_lambda(a, b, c) == pytest.approx(lam, abs=1e-15)
        assert oracle_mod.line_dist2(a, b, c, lam) == pytest.approx(d2, abs=1e-12)


def test_eq7_equals_distance_to_anchor_for_any_lambda(oracle_mod):
    rng = np.random.default_rng(7)
    for _ in range(200):
        D = int(rng.integers(1, 40))
        ci, cj, x = rng.normal(size=(3, D)) * rng.uniform(0.1, 50)
        lam = rng.uniform(-2, 3)
        a, b, c = ((x - ci) ** 2).sum(), ((x - cj) ** 2).sum(), ((cj - ci) ** 2).sum()
        direct = ((x - ((1 - lam) * ci + lam * cj)) ** 2).sum()
        assert oracle_mod.line_dist2(a, b, c, lam) == pytest.approx(direct, rel=1e-10, abs=1e-10)


def test_eq8_is_the_orthogonal_projection(oracle_mod):
    rng = np.random.default_rng(8)
    for _ in range(200):
        D = int(rng.integers(2, 40))
        ci, cj, x = rng.normal(size=(3, D)) * 10
        a, b, c = ((x - ci) ** 2).sum(), ((x - cj) ** 2).sum(), ((cj - ci) ** 2).sum()
        lam = oracle_mod.line_lambda(a, b, c)
        # least squares: min_l |(x - ci) - l (cj - ci)|
        sol, res, *_ = np.linalg.lstsq((cj - ci)[:, None], x - ci, rcond=None)
        assert lam == pytest.approx(sol[0], rel=1e-9, abs=1e-12)
        d2 = oracle_mod.line_dist2(a, b, c, lam)
        assert d2 == pytest.approx(res[0], rel=1e-8, abs=1e-9)
        assert d2 == pytest.approx(a - c * lam * lam, rel=1e-9, abs=1e-9)
        # a minimum: moving along the line only increases the distance
        for dl in (-1e-3, 1e-3):
            assert oracle_mod.line_dist2(a, b, c, lam + dl) >= d2
        # residual orthogonal to the line direction
        anchor = (1 - lam) * ci + lam * cj
        assert abs(np.dot(x - anchor, cj - ci)) < 1e-8 * (1 + c)


def test_duplicate_centroids_give_lambda_zero(oracle_mod):
    assert oracle_mod.line_lambda(3.0, 3.0, 0.0) == 0.0
    assert oracle_mod.line_dist2(3.0, 3.0, 0.0, 0.0) == 3.0


# ---- lambda byte -----------------------------------------------------------


def test_lambda_grid(oracle_mod):
    o = oracle_mod
    assert o.lambda_quant(0.0) == 85 and o.lambda_dequant(85) == 0.0
    assert o.lambda_quant(0.5) == 255 and o.lambda_dequant(255) == pytest.approx(0.5, abs=1e-15)
    assert o.lambda_quant(-0.25) == 0 and o.lambda_dequant(0) == pytest.approx(-0.25, abs=1e-15)
    assert o.lambda_quant(7.0) == 255 and o.lambda_quant(-7.0) == 0
    step = 0.75 / 255
    assert step == pytest.approx(1 / 340)
    # half-way cases go to the even code
    assert o.lambda_quant(0.5 * step) == 85 + 0  # 85.5 -> 86? no: rint(0.5)=0 -> 85
    assert o.lambda_quant(1.5 * step) == 85 + 2
    assert o.lambda_quant(-0.5 * step) == 85
    rng = np.random.default_rng(3)
    for lam in rng.uniform(-0.25, 0.5, 500):
        q = o.lambda_quant(lam)
        assert abs(o.lambda_dequant(q) - lam) <= step / 2 + 1e-12
        assert o.lambda_coord(lam) == pytest.approx(lam * 340 + 85, abs=1e-9)
    # another grid with 0 on it
    # step 1.5 / 255 = 1 / 170: zero is code 170, 0.5 is code 255, -1 is code 0
    assert o.lambda_quant(0.0, -1.0, 0.5) == 170 and o.lambda_dequant(170, -1.0, 0.5) == 0.0
    assert o.lambda_quant(0.5, -1.0, 0.5) == 255 and o.lambda_quant(-1.0, -1.0, 0.5) == 0
    assert o.lambda_dequant(0, -1.0, 0.5) == pytest.approx(-1.0, abs=1e-15)
    assert o.lambda_coord(0.25, -1.0, 0.5) == pytest.approx(170 + 42.5, abs=1e-9) and o.lambda_quant(0.25, -1.0, 0.5) == 212


# ---- graph -----------------------------------------------------------------


def test_graph_against_cdist(oracle_mod):
    pr = problem(k=40, n=6, N=1000)
    S, E = oracle_mod.graph(pr.C, 6)
    d = cdist(pr.C.astype(np.float64), pr.C.astype(np.float64), "sqeuclidean")
    np.fill_diagonal(d, np.inf)
    order = np.argsort(d, axis=1, kind="stable")[:, :6]
    assert (S == order).all()
    assert np.allclose(E, np.take_along_axis(d, order, 1), rtol=1e-12)
    assert (S != np.arange(40)[:, None]).all()
    # rows on demand agree with the full graph
    S2, E2 = oracle_mod.graph(pr.C, 6, rows=[5, 17, 3])
    assert (S2 == S[[5, 17, 3]]).all() and (E2 == E[[5, 17, 3]]).all()


def test_select_smallest_ties_go_to_smaller_key(oracle_mod):
    val = np.array([[3.0, 1.0, 1.0, 2.0, 1.0]])
    assert oracle_mod.select_smallest(val, 4).tolist() == [[1, 2, 4, 3]]
    key = np.array([[50, 40, 30, 20, 10]], np.int32)
    assert oracle_mod.select_smallest(val, 4, key).tolist() == [[10, 30, 40, 20]]
    assert oracle_mod.select_smallest(val, 7).tolist() == [[1, 2, 4, 3, 0, -1, -1]]
    rng = np.random.default_rng(0)
    v = rng.integers(0, 5, (20, 30)).astype(np.float64)
    got = oracle_mod.select_smallest(v, 9)
    want = np.stack([np.lexsort((np.arange(30), r))[:9] for r in v])
    assert (got == want).all()


# ---- encoding: brute force over every choice on tiny inputs ---------------


def _encode_bruteforce(pr, S, lo=-0.25, hi=0.5):
    """Alg. 1 + Alg. 2 from vector algebra only (no a/b/c formulae)."""
    X, Cb, P = pr.X.astype(np.float64), pr.C.astype(np.float64), pr.P.astype(np.float64)
    m, ds = pr.m, pr.D // pr.m
    step = (hi - lo) / 255
    zero = -round(lo / step)
    cell = cdist(X, Cb, "sqeuclidean").argmin(1)
    edge = np.zeros(len(X), int)
    lamq = np.zeros(len(X), int)
    codes = np.zeros((len(X), m), int)
    lam_real = np.zeros(len(X))
    for t, x in enumerate(X):
        ci = Cb[cell[t]]
        best = None
        for j in range(pr.n):
            e = Cb[S[cell[t], j]] - ci
            lam = np.dot(x - ci, e) / np.dot(e, e)
            d2 = ((x - ci - lam * e) ** 2).sum()
            if best is None or d2 < best[0]:
                best = (d2, j, lam)
        edge[t], lam_real[t] = best[1], best[2]
        q = int(np.clip(np.rint(best[2] / step) + zero, 0, 255))
        lamq[t] = q
        lh = (q - zero) * step
        r = x - ((1 - lh) * ci + lh * Cb[S[cell[t], best[1]]])
        for p in range(m):
            codes[t, p] = cdist(r[None, p * ds:(p + 1) * ds], P[p], "sqeuclidean").argmin()
    return cell, edge, lamq, codes, lam_real


@pytest.mark.parametrize("cfg", [dict(N=300, k=6, n=3, D=4, m=2, G=3), dict(N=400, k=16, n=4, D=8, m=2, G=5),
                                 dict(kind="deep", N=300, k=12, n=4, D=12, m=4, G=4)])
def test_encode_against_bruteforce(oracle_mod, cfg):
    pr = problem(nq=5, iters=3, **cfg)
    S, E = oracle_mod.graph(pr.C, pr.n)
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    cell, edge, lamq, codes, lam_real = _encode_bruteforce(pr, S)
    assert (enc.cell == cell).all()
    assert (enc.edge == edge).all()
    assert np.allclose((enc.lam_coord - 85) / 340, lam_real, atol=1e-9)
    assert (enc.lamq == lamq).all()
    assert (enc.codes == codes).all()
    # diagnostics are what they claim
    d = cdist(pr.X.astype(np.float64), pr.C.astype(np.float64), "sqeuclidean")
    ds = np.sort(d, 1)
    assert np.allclose(enc.cell_d, ds[:, :2], rtol=1e-12)
    assert (enc.edge_d[:, 0] <= enc.edge_d[:, 1]).all() and (enc.code_d[..., 0] <= enc.code_d[..., 1]).all()


def test_vq_assign_matches_encode(oracle_mod):
    pr = problem(N=500, k=16, n=4, D=8, m=2, G=5, nq=5, iters=3)
    S, E = oracle_mod.graph(pr.C, pr.n)
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    cell, cd = oracle_mod.vq_assign(pr.C, pr.X)
    assert (cell == enc.cell).all() and (cd == enc.cell_d).all()
    # a sparse graph holding only the needed rows encodes identically
    S2, E2 = oracle_mod.sparse_graph(pr.C, pr.n, cell)
    enc2 = oracle_mod.encode(pr.C, S2, E2, pr.P, pr.X)
    assert (enc2.edge == enc.edge).all() and (enc2.codes == enc.codes).all() and (enc2.lamq == enc.lamq).all()


@pytest.mark.parametrize("kind,D,m", [("sift", 128, 8), ("deep", 96, 16)])
def test_lambda_range_and_anchor_error(oracle_mod, kind, D, m):
    """A point of cell i has a <= b for every edge, hence lambda <= 1/2 and
    |lambda| <= sqrt(a/c) (Eq. 8); with 0 on the byte grid the anchor is never
    farther from x than c_i is (the claim under Fig. 1c, Sec. 3.2)."""
    pr = problem(kind=kind, N=3000, k=48, n=8, m=m, G=24, nq=5)
    S, E = oracle_mod.graph(pr.C, pr.n)
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    lam = (enc.lam_coord - 85) / 340
    assert (lam <= 0.5 + 1e-12).all()
    a = enc.cell_d[:, 0]
    c = E[enc.cell, enc.edge]
    assert (np.abs(lam) <= np.sqrt(a / c) + 1e-12).all()
    assert (enc.lamq[lam >= 0] >= 85).all() and (enc.lamq[lam <= 0] <= 85).all()
    X, Cb = pr.X.astype(np.float64), pr.C.astype(np.float64)
    lh = (enc.lamq.astype(np.float64) - 85) / 340
    ci, sj = Cb[enc.cell], Cb[S[enc.cell, enc.edge]]
    anchor = (1 - lh)[:, None] * ci + lh[:, None] * sj
    err_anchor = ((X - anchor) ** 2).sum(1)
    assert (err_anchor <= a * (1 + 1e-12) + 1e-12).all()
    assert err_anchor.mean() < a.mean()  # and it does help on average
    # edge_d[:,0] is the unquantised line distance a - c lambda^2
    assert np.allclose(enc.edge_d[:, 0], a - c * lam * lam, rtol=1e-9, atol=1e-9)


# ---- search ----------------------------------------------------------------


def _index(oracle_mod, pr, force_lambda_zero=False):
    S, E = oracle_mod.graph(pr.C, pr.n)
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    lamq = np.full_like(enc.lamq, 85) if force_lambda_zero else enc.lamq
    lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, lamq, enc.codes)
    return S, E, enc, lists


def _reconstruct_numpy(pr, S, cell, edge, lamq, codes):
    Cb, P = pr.C.astype(np.float64), pr.P.astype(np.float64)
    lh = (lamq.astype(np.float64) - 85) / 340
    q1 = (1 - lh)[:, None] * Cb[cell] + lh[:, None] * Cb[S[cell, edge]]
    q2 = np.concatenate([P[p][codes[:, p]] for p in range(pr.m)], axis=1)
    return q1 + q2, q1, q2


def test_make_lists_layout(oracle_mod):
    pr = problem(N=800, k=12, n=3, D=8, m=2, G=4, nq=4, iters=3)
    S, E, enc, lists = _index(oracle_mod, pr)
    assert lists.off[0] == 0 and lists.off[-1] == 800 and len(lists.off) == 12 * 3 + 1
    for l in range(36):
        ids = lists.ids[lists.off[l]:lists.off[l + 1]]
        assert (np.diff(ids) > 0).all()
        assert ((enc.cell[ids] * 3 + enc.edge[ids]) == l).all()
        assert (lists.codes[lists.off[l]:lists.off[l + 1]] == enc.codes[ids]).all()
        assert (lists.lamq[lists.off[l]:lists.off[l + 1]] == enc.lamq[ids]).all()


def test_exhaustive_probe_is_bruteforce_over_reconstructions(oracle_mod):
    pr = problem(N=1500, k=16, n=4, m=8, G=8, nq=20, D=32)
    S, E, enc, lists = _index(oracle_mod, pr)
    tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=pr.k, w2=pr.k * pr.n, K=25)
    Xh, _, _ = _reconstruct_numpy(pr, S, enc.cell, enc.edge, enc.lamq, enc.codes)
    assert np.allclose(oracle_mod.reconstruct(pr.C, S, pr.P, enc.cell, enc.edge, enc.lamq, enc.codes), Xh, rtol=1e-13)
    d = cdist(pr.Y.astype(np.float64), Xh, "sqeuclidean")
    order = np.stack([np.lexsort((np.arange(d.shape[1]), r))[:25] for r in d])
    assert (tr.ncand == 1500).all()
    assert np.allclose(tr.out_d, np.take_along_axis(d, order, 1), rtol=1e-10)
    assert (tr.out_id == order).all()


def test_scan_distance_equals_the_paper_decomposition(oracle_mod):
    """Eq. 14 == Eq. 16 with term1 expanded by Eq. 17, term by term."""
    pr = problem(N=1200, k=16, n=4, m=8, G=8, nq=12, D=32)
    S, E, enc, lists = _index(oracle_mod, pr)
    tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=6, w2=10, K=40)
    Cb, Y = pr.C.astype(np.float64), pr.Y.astype(np.float64)
    Xh, q1, q2 = _reconstruct_numpy(pr, S, enc.cell, enc.edge, enc.lamq, enc.codes)
    lh = (enc.lamq.astype(np.float64) - 85) / 340
    for q in range(len(Y)):
        for d, t in zip(tr.out_d[q], tr.out_id[q]):
            if t < 0:
                continue
            i, j = enc.cell[t], enc.edge[t]
            ci, sij, y, lam = Cb[i], Cb[S[i, j]], Y[q], lh[t]
            term6, term7, term8 = ((y - ci) ** 2).sum(), ((ci - sij) ** 2).sum(), ((y - sij) ** 2).sum()
            term1 = (1 - lam) * term6 + (lam * lam - lam) * term7 + lam * term8
            term2 = (q2[t] ** 2).sum()
            term3, term4, term5 = ci @ q2[t], sij @ q2[t], 2 * (y @ q2[t])
            assert d == pytest.approx(term1 + term2 + 2 * (1 - lam) * term3 + 2 * lam * term4 - term5, rel=1e-9)


def test_traversal_steps(oracle_mod):
    """Region traversal (Sec. 3.3.1): cells by coarse distance, sub-regions by the
    query's own distance to each line, computed here by explicit projection."""
    pr = problem(N=1200, k=16, n=4, m=8, G=8, nq=12, D=32)
    S, E, enc, lists = _index(oracle_mod, pr)
    w1, w2 = 5, 7
    tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=w1, w2=w2, K=10)
    Cb, Y = pr.C.astype(np.float64), pr.Y.astype(np.float64)
    d = cdist(Y, Cb, "sqeuclidean")
    assert np.allclose(tr.dist, d, rtol=1e-12)
    assert (tr.cells == np.argsort(d, 1, kind="stable")[:, :w1]).all()
    for q in range(len(Y)):
        sc = []
        for i in tr.cells[q]:
            for j in range(pr.n):
                e = Cb[S[i, j]] - Cb[i]
                lam = np.dot(Y[q] - Cb[i], e) / np.dot(e, e)
                sc.append((((Y[q] - Cb[i] - lam * e) ** 2).sum(), i * pr.n + j))
        assert np.allclose(tr.score[q], [s for s, _ in sc], rtol=1e-8, atol=1e-8)
        assert (tr.label[q] == [l for _, l in sc]).all()
        # l(c_i, c_j) and l(c_j, c_i) are the same geometric line, so exact ties are
        # common: compare the selected scores, and the labels up to such ties
        want = sorted(sc)
        got_sc = {l: s for s, l in sc}
        assert np.allclose([got_sc[l] for l in tr.sub[q]], [s for s, _ in want[:w2]], rtol=1e-9, atol=1e-9)
        cut = want[w2 - 1][0]
        sure = {l for s, l in want if s < cut * (1 - 1e-9) - 1e-9}
        assert sure <= set(tr.sub[q].tolist()) and len(set(tr.sub[q].tolist())) == w2
        # with its own scores the oracle's choice is exactly the (score, label) order
        mine = sorted(zip(tr.score[q].tolist(), tr.label[q].tolist()))[:w2]
        assert tr.sub[q].tolist() == [l for _, l in mine]
        # candidates = exactly the points stored in the visited lists
        assert tr.ncand[q] == sum(lists.off[l + 1] - lists.off[l] for l in tr.sub[q])


@pytest.mark.parametrize("qlam", [(0.0, 1.0), (-0.25, 0.5), (0.3, 0.3)])
def test_restricted_query_lambda_is_the_distance_to_the_segment(oracle_mod, qlam):
    """Sec. 3.3.1 variant: with the query's lambda restricted to [lo, hi] the score of a sub-region is
    the squared distance from the query to that segment of the line.  Checked against a dense sampling
    of the segment (no a / b / c formulae), and against the unrestricted scores where the foot of the
    perpendicular already lies inside the range."""
    pr = problem(N=1200, k=16, n=4, m=8, G=8, nq=12, D=32)
    S, E = oracle_mod.graph(pr.C, pr.n)
    Cb, Y = pr.C.astype(np.float64), pr.Y.astype(np.float64)
    dist = oracle_mod.coarse(pr.C, pr.Y)
    cells = oracle_mod.select_smallest(dist, 5)
    free, label0 = oracle_mod.subregion_scores(dist, S, E, cells)
    got, label = oracle_mod.subregion_scores(dist, S, E, cells, qlam)
    assert (label == label0).all() and (got >= free - 1e-9 * np.abs(free)).all()
    lo, hi = qlam
    ts = np.linspace(lo, hi, 20001)
    inside = outside = 0
    for q in range(len(Y)):
        o = 0
        for i in cells[q]:
            for j in range(pr.n):
                e = Cb[S[i, j]] - Cb[i]
                z = Y[q] - Cb[i]
                # ||z - t e||^2 over the sampled segment
                sampled = ((z @ z) - 2 * ts * (z @ e) + ts * ts * (e @ e)).min()
                step_err = (e @ e) * ((hi - lo) / 20000) ** 2  # the sampling misses the minimum by at most half a step
                assert sampled - step_err - 1e-9 * sampled <= got[q, o] <= sampled + 1e-9 * sampled, (q, i, j)
                lam = (z @ e) / (e @ e)
                if lo <= lam <= hi:
                    assert got[q, o] == pytest.approx(free[q, o], rel=1e-12)
                    inside += 1
                else:
                    end = lo if lam < lo else hi
                    assert got[q, o] == pytest.approx(((z - end * e) ** 2).sum(), rel=1e-9)
                    assert got[q, o] > free[q, o]
                    outside += 1
                o += 1
    assert outside > 20 and (inside > 20 or lo == hi)


def _ivfadc(pr, cell, codes, Y, w, K):
    """Textbook IVFADC (Sec. 2.3): probe the w nearest cells, score residual PQ
    codes through per-cell lookup tables, keep the K best."""
    Cb, P = pr.C.astype(np.float64), pr.P.astype(np.float64)
    m, ds = pr.m, pr.D // pr.m
    out_d, out_i = [], []
    for y in Y.astype(np.float64):
        probe = np.argsort(((Cb - y) ** 2).sum(1), kind="stable")[:w]
        cand = []
        for i in probe:
            r = y - Cb[i]
            tab = np.stack([((P[p] - r[p * ds:(p + 1) * ds]) ** 2).sum(1) for p in range(m)])
            for t in np.nonzero(cell == i)[0]:
                cand.append((sum(tab[p, codes[t, p]] for p in range(m)), t))
        cand.sort()
        out_d.append([c[0] for c in cand[:K]])
        out_i.append([c[1] for c in cand[:K]])
    return np.array(out_d), np.array(out_i)


def test_lambda_zero_reduces_to_ivfadc(oracle_mod):
    pr = problem(N=1500, k=16, n=4, m=8, G=8, nq=15, D=32)
    S, E = oracle_mod.graph(pr.C, pr.n)
    # residuals w.r.t. the centroid itself: encode with a grid whose only reachable value is 0
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    cell = enc.cell
    X, Cb, P = pr.X.astype(np.float64), pr.C.astype(np.float64), pr.P.astype(np.float64)
    ds = pr.D // pr.m
    R = X - Cb[cell]
    codes = np.stack([cdist(R[:, p * ds:(p + 1) * ds], P[p], "sqeuclidean").argmin(1) for p in range(pr.m)], 1).astype(np.uint8)
    lists = oracle_mod.make_lists(pr.k, pr.n, cell, enc.edge, np.full(len(X), 85, np.uint8), codes)
    w1, K = 5, 30
    tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=w1, w2=w1 * pr.n, K=K)
    d, i = _ivfadc(pr, cell, codes, pr.Y, w1, K)
    assert (tr.out_id == i).all()
    assert np.allclose(tr.out_d, d, rtol=1e-9)


def test_exactly_representable_data_gives_exact_knn(oracle_mod):
    """Points built as anchor(grid lambda) + tiny codewords are reproduced exactly,
    so exhaustive probing must equal exact k-NN on the raw vectors."""
    rng = np.random.default_rng(5)
    k, n, D, m, N = 10, 3, 8, 2, 400
    ds = D // m
    Cb = (rng.normal(size=(k, D)) * 100).astype(np.float32)
    P = (rng.normal(size=(m, 256, ds)) * 1e-3).astype(np.float32)
    S, E = oracle_mod.graph(Cb, n)
    cell = rng.integers(0, k, N)
    edge = rng.integers(0, n, N)
    lamq = rng.integers(60, 110, N)  # small |lambda|: x stays inside its cell and nearest to its line
    codes = rng.integers(0, 256, (N, m))
    lh = (lamq - 85) / 340
    Cd = Cb.astype(np.float64)
    X = (1 - lh)[:, None] * Cd[cell] + lh[:, None] * Cd[S[cell, edge]]
    X += np.concatenate([P[p][codes[:, p]] for p in range(m)], 1)
    # make x exactly representable in fp32 so that both sides see the same numbers
    X32 = X.astype(np.float32)
    enc = oracle_mod.encode(Cb, S, E, P, X32)
    assert (enc.cell == cell).all()
    Xh = oracle_mod.reconstruct(Cb, S, P, enc.cell, enc.edge, enc.lamq, enc.codes)
    assert np.abs(Xh - X32).max() < 5e-3  # within a codeword of the original
    lists = oracle_mod.make_lists(k, n, enc.cell, enc.edge, enc.lamq, enc.codes)
    Y = (X32[rng.integers(0, N, 12)] + rng.normal(size=(12, D)) * 30).astype(np.float32)
    tr = oracle_mod.search(Cb, S, E, P, lists, Y, w1=k, w2=k * n, K=10)
    d = cdist(Y.astype(np.float64), X32.astype(np.float64), "sqeuclidean")
    want = np.argsort(d, 1, kind="stable")[:, :10]
    # neighbours are separated by far more than the codeword-sized reconstruction error
    assert (tr.out_id == want).all()


def test_recall_monotone_in_K_and_w2(oracle_mod):
    pr = problem(N=4000, k=32, n=4, m=8, G=16, nq=50)
    S, E, enc, lists = _index(oracle_mod, pr)
    nn = cdist(pr.Y.astype(np.float64), pr.X.astype(np.float64), "sqeuclidean").argmin(1)
    prev = -1.0
    for w2 in (4, 8, 16, 32):
        tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=8, w2=w2, K=50)
        found = [(tr.out_id[:, :K] == nn[:, None]).any(1).mean() for K in (1, 10, 50)]
        assert found[0] <= found[1] <= found[2]
        # the candidate set only grows with w2, so the true neighbour is never lost again
        cover = np.mean([nn[q] in set(np.concatenate([lists.ids[lists.off[l]:lists.off[l + 1]] for l in tr.sub[q]])) for q in range(50)])
        assert cover >= prev
        prev = cover
    assert prev > 0.5


def test_short_rows_are_padded(oracle_mod):
    pr = problem(N=300, k=6, n=3, D=4, m=2, G=3, nq=5, iters=3)
    S, E, enc, lists = _index(oracle_mod, pr)
    tr = oracle_mod.search(pr.C, S, E, pr.P, lists, pr.Y, w1=1, w2=1, K=400)
    for q in range(5):
        nc = tr.ncand[q]
        assert nc < 400
        assert np.isinf(tr.out_d[q, nc:]).all() and (tr.out_id[q, nc:] == -1).all()
        assert np.isfinite(tr.out_d[q, :nc]).all() and (np.diff(tr.out_d[q, :nc]) >= 0).all()


# ---- printed constants (Sec. 3.1; Sec. 5 memory paragraph, Table 4) --------


def test_memory_figures(oracle_mod):
    assert oracle_mod.graph_bytes(2 ** 16, 32) == 16 * 2 ** 20  # "16 MB"
    assert oracle_mod.second_level_vq_bytes(2 ** 16, 32, 128) == 1024 * 2 ** 20  # "1,024 MB"
    assert oracle_mod.second_level_vq_bytes(2 ** 16, 32, 128) // oracle_mod.graph_bytes(2 ** 16, 32) == 64  # "1/64"
    # Table 4 prints 13.55 GB for k = 2^16; the formula gives that to 0.1 GB with n = 32
    assert oracle_mod.index_bytes(10 ** 9, 2 ** 16, 32, 128, 8) / 1e9 == pytest.approx(13.55, abs=0.1)


# ---------------------------------------------------------------------------
# training helpers (Sec. 2.1 / Sec. 5: codebooks by k-means; Eq. 12 residuals)
# ---------------------------------------------------------------------------
def test_lloyd_step_hand_example_and_textbook_routine(oracle_mod):
    # four points on a line, two centroids: {0, 1} and {10, 11} -> means 0.5 and 10.5
    X = np.array([[0.0], [1.0], [10.0], [11.0]], np.float32)
    C0 = np.array([[0.0], [10.0]], np.float32)
    C1, cell, _ = oracle_mod.lloyd_step(C0, X)
    assert cell.tolist() == [0, 0, 1, 1] and np.allclose(C1[:, 0], [0.5, 10.5])
    # a centroid without members stays; an exact tie goes to the smaller index
    C0 = np.array([[0.0], [2.0], [100.0]], np.float32)
    X = np.array([[1.0], [-1.0]], np.float32)
    C1, cell, _ = oracle_mod.lloyd_step(C0, X)
    assert cell.tolist() == [0, 0] and np.allclose(C1[:, 0], [0.0, 2.0, 100.0])
    # against scikit-learn's Lloyd, one iteration from the same initial centroids
    from sklearn.cluster import KMeans

    rng = np.random.default_rng(5)
    X = rng.normal(size=(3000, 12)).astype(np.float32) + rng.integers(0, 6, size=(3000, 1)).astype(np.float32) * 3
    C0 = X[rng.choice(3000, 40, replace=False)].copy()
    C1, cell, _ = oracle_mod.lloyd_step(C0, X)
    km = KMeans(n_clusters=40, init=C0.astype(np.float64), n_init=1, max_iter=1, algorithm="lloyd", tol=0.0).fit(X.astype(np.float64))
    assert np.allclose(km.cluster_centers_, C1, rtol=1e-6, atol=1e-6)
    # the k-means objective never increases from one iteration to the next
    obj = []
    Cc = C0.astype(np.float64)
    for _ in range(4):
        Cn, cell, cd = oracle_mod.lloyd_step(Cc.astype(np.float32), X)
        obj.append(cd[:, 0].sum())
        Cc = Cn
    assert all(b <= a * (1 + 1e-6) for a, b in zip(obj, obj[1:]))


def test_line_residual_is_the_vector_from_the_anchor(oracle_mod):
    pr = problem(N=600, k=16, n=4, m=4, G=4, nq=5, D=8)
    S, E = oracle_mod.graph(pr.C, pr.n)
    enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
    R = oracle_mod.line_residual(pr.C, S, pr.X, enc.cell, enc.edge, enc.lamq)
    # anchor + residual gives the vector back; reconstruct() = anchor + codewords, so
    # x - reconstruct = residual - codewords
    cw = np.stack([pr.P[p][enc.codes[:, p]] for p in range(pr.m)], 1).reshape(len(pr.X), -1)
    Xh = oracle_mod.reconstruct(pr.C, S, pr.P, enc.cell, enc.edge, enc.lamq, enc.codes)
    assert np.allclose(pr.X - Xh, R - cw, atol=1e-9)
    # the anchor lies on the line through c_i and s_ij: (x - r - c_i) is parallel to (s_ij - c_i)
    anchor = pr.X - R
    v = anchor - pr.C[enc.cell]
    e = pr.C[S[enc.cell, enc.edge]] - pr.C[enc.cell]
    cross = (v * v).sum(1) * (e * e).sum(1) - ((v * e).sum(1)) ** 2
    assert (np.abs(cross) <= 1e-6 * (1 + (v * v).sum(1) * (e * e).sum(1))).all()
    # and never farther from x than the centroid (the grid contains 0)
    assert ((R * R).sum(1) <= ((pr.X - pr.C[enc.cell]) ** 2).sum(1) * (1 + 1e-9) + 1e-9).all()
