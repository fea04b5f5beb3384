"""GPU library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from parity import DTOL, EPS32, GAP, LAM_WINDOW, RES_ROUNDINGS, check_selection, check_topk, term_scale
from util import Problem, problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vlq():
    import paper_1901_00275_amd as vlq

    vlq.lib()
    assert torch.cuda.is_available()
    return vlq


DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def make_index(vlq, pr, base=None, lo=0.0, hi=0.0):
    prm = vlq.vlq_params_t(pr.D, pr.k, pr.n, pr.m, lo, hi)
    if base is None:
        return vlq.vlq_build_index(prm, dev(pr.C), dev(pr.P))
    return vlq.vlq_build_index(prm, dev(pr.C), dev(pr.P), dev(base), base.shape[0])


def gpu_graph(vlq, idx, pr):
    S = torch.empty(pr.k, pr.n, dtype=torch.int32, device=DEV)
    E = torch.empty(pr.k, pr.n, dtype=torch.float32, device=DEV)
    vlq.vlq_index_get_graph(idx, S, E)
    torch.cuda.synchronize()
    return S.cpu().numpy(), E.cpu().numpy()


def check_graph(oracle, pr, Sg, Eg):
    So, Eo = oracle.graph(pr.C, min(pr.n + 1, pr.k - 1))
    same = True
    Cd = pr.C.astype(np.float64)
    for i in range(pr.k):
        if (Sg[i] == So[i, : pr.n]).all():
            continue
        d = ((Cd - Cd[i]) ** 2).sum(1)
        val = {j: d[j] for j in range(pr.k) if j != i}
        same &= check_selection(Sg[i], val, pr.n, what=f"graph row {i}")
    dg = ((Cd[Sg] - Cd[:, None, :]) ** 2).sum(2)
    assert np.allclose(Eg, dg, rtol=DTOL)
    return same


def gpu_encode(vlq, idx, X, m):
    nb = X.shape[0]
    cell = torch.empty(nb, dtype=torch.int32, device=DEV)
    edge = torch.empty(nb, dtype=torch.int32, device=DEV)
    lam = torch.empty(nb, dtype=torch.uint8, device=DEV)
    codes = torch.empty(nb, m, dtype=torch.uint8, device=DEV)
    vlq.vlq_encode(idx, dev(X), nb, cell, edge, lam, codes)
    torch.cuda.synchronize()
    return cell.cpu().numpy(), edge.cpu().numpy(), lam.cpu().numpy(), codes.cpu().numpy()


def check_encode(oracle, pr, S, E, X, got, max_soft=0.01, grid=()):
    """Stage by stage; a point whose upstream choice differs inside the tie band is
    not compared further downstream (counted instead)."""
    cell, edge, lamq, codes = got
    enc = oracle.encode(pr.C, S, E, pr.P, X, *grid)
    N = len(X)
    soft = 0
    ok = np.ones(N, bool)
    # VQ (Eq. 2): gap relative to the distance
    bad = np.nonzero(cell != enc.cell)[0]
    for t in bad:
        assert enc.cell_d[t, 1] - enc.cell_d[t, 0] <= GAP * enc.cell_d[t, 1], f"cell of point {t}"
        dg = ((X[t].astype(np.float64) - pr.C[cell[t]].astype(np.float64)) ** 2).sum()
        assert dg <= enc.cell_d[t, 0] * (1 + GAP) + 1e-30
    ok[bad] = False
    soft += len(bad)
    # LQ (Alg. 1): gap relative to a, because a - c lambda^2 cancels
    bad = np.nonzero(ok & (edge != enc.edge))[0]
    for t in bad:
        assert enc.edge_d[t, 1] - enc.edge_d[t, 0] <= GAP * max(enc.cell_d[t, 0], 1e-30), f"edge of point {t}"
    ok[bad] = False
    soft += len(bad)
    # lambda byte: equal, or one step apart when the coordinate sits on a rounding boundary
    bad = np.nonzero(ok & (lamq != enc.lamq))[0]
    for t in bad:
        assert abs(int(lamq[t]) - int(enc.lamq[t])) == 1, f"lambda byte of point {t}"
        frac = enc.lam_coord[t] - np.floor(enc.lam_coord[t])
        assert abs(frac - 0.5) < LAM_WINDOW, f"lambda byte of point {t}: coordinate {enc.lam_coord[t]}"
    ok[bad] = False
    soft += len(bad)
    # PQ (Alg. 2): gap relative to the sub-space distance
    diff = (codes != enc.codes) & ok[:, None]
    ds = pr.D // pr.m
    for t, p in zip(*np.nonzero(diff)):
        d0, d1 = enc.code_d[t, p]
        if d1 - d0 <= GAP * max(d1, 1e-30) + 1e-12:
            continue
        # the residual itself is only known to its rounding to fp32
        rp = oracle.line_residual(pr.C, S, X[t:t + 1], enc.cell[t:t + 1], enc.edge[t:t + 1], enc.lamq[t:t + 1],
                                  *grid)[0, p * ds:(p + 1) * ds]
        dr = RES_ROUNDINGS * EPS32 * np.linalg.norm(rp)
        assert np.sqrt(d1) - np.sqrt(d0) <= dr, f"code of point {t}, sub-space {p}"
    soft += int(diff.any(1).sum())
    assert soft <= max(2, max_soft * N), f"{soft} of {N} points fell into tie bands"
    return enc, soft


def load_oracle_index(vlq, idx, enc, ids=None):
    N = len(enc.cell)
    vlq.vlq_index_add_encoded(idx, dev(enc.cell), dev(enc.edge), dev(enc.lamq), dev(enc.codes),
                              None if ids is None else dev(ids, torch.int32), N)
    vlq.vlq_index_finalize(idx)


def gpu_search(vlq, idx, Y, w1, w2, K):
    nq = Y.shape[0]
    od = torch.empty(nq, K, device=DEV)
    oi = torch.empty(nq, K, dtype=torch.int32, device=DEV)
    cells = torch.empty(nq, w1, dtype=torch.int32, device=DEV)
    cd = torch.empty(nq, w1, device=DEV)
    sub = torch.empty(nq, w2, dtype=torch.int32, device=DEV)
    ss = torch.empty(nq, w2, device=DEV)
    vlq.vlq_search_debug(idx, dev(Y), nq, w1, w2, K, od, oi, cells, cd, sub, ss)
    torch.cuda.synchronize()
    od2 = torch.empty(nq, K, device=DEV)
    oi2 = torch.empty(nq, K, dtype=torch.int32, device=DEV)
    vlq.vlq_search(idx, dev(Y), nq, w1, w2, K, od2, oi2)
    torch.cuda.synchronize()
    assert torch.equal(oi, oi2) and torch.equal(od, od2)  # deterministic, debug == plain
    return [t.cpu().numpy() for t in (od, oi, cells, cd, sub, ss)]


def check_search(oracle, pr, S, E, lists, Y, w1, w2, K, got, max_soft=0.15, grid=(), qlam=(-np.inf, np.inf)):
    """Stage by stage.  Where the oracle itself sees a tie (mirrored lines
    l(c_i,c_j) / l(c_j,c_i) tie exactly in exact arithmetic) the GPU's choice is
    first checked to lie inside the oracle's tie band, then the next stage is
    compared for that choice."""
    od, oi, cells, cd, sub, ss = got
    extra = 16
    lo_hi = grid if grid else (oracle.LAMBDA_LO, oracle.LAMBDA_HI)
    tr = oracle.search(pr.C, S, E, pr.P, lists, Y, w1, w2, K + extra, *lo_hi, qlam=qlam)
    nq = len(Y)
    soft = 0
    for q in range(nq):
        what = f"query {q}"
        same_cells = check_selection(cells[q], dict(enumerate(tr.dist[q])), w1, what=what + " cells")
        assert np.allclose(cd[q], tr.dist[q][cells[q]], rtol=DTOL), what
        score, label = tr.score[q], tr.label[q]
        if not same_cells:
            score, label = (x[0] for x in oracle.subregion_scores(tr.dist[q:q + 1], S, E, cells[q:q + 1], qlam))
        a_max = tr.dist[q][cells[q]].max()
        val = {int(l): float(s) for l, s in zip(label, score)}
        same_sub = check_selection(sub[q], val, w2, scale=a_max, what=what + " sub-regions")
        assert np.allclose(ss[q], [val[int(l)] for l in sub[q]], rtol=0, atol=DTOL * a_max), what
        o_d, o_i = tr.out_d[q], tr.out_id[q]
        if not (same_cells and same_sub):
            soft += 1
            o_d, o_i, _ = (x[0] for x in oracle.scan(pr.C, S, pr.P, lists, Y[q:q + 1], sub[q:q + 1], K + extra, *grid))
        check_topk(od[q], oi[q], o_d, o_i, K, what=what, scale=term_scale(a_max, Y[q], pr.C, pr.P), m=pr.m)
    assert soft <= max(3, max_soft * nq), f"{soft} of {nq} queries fell into tie bands"
    return tr, soft


def shifted(pr, shift):
    """The same problem with data, queries and centroids moved by one vector (codewords quantise
    residuals and stay): every distance is unchanged in exact arithmetic."""
    if not shift:
        return pr
    v = np.float32(shift)
    return Problem(pr.kind, pr.X + v, pr.Y + v, pr.C + v, pr.P, pr.n)


CASES = {
    # name: (problem kwargs, w1, w2, K[, shift])
    "small_d32": (dict(N=3000, k=32, n=4, m=8, G=8, nq=40, D=32), 6, 10, 20),
    "sift_ragged": (dict(N=20011, k=100, n=7, m=8, G=16, nq=77), 9, 25, 100),
    "deep_m16": (dict(kind="deep", N=15000, k=96, n=8, m=16, G=32, nq=50), 8, 20, 50),
    "odd_dims": (dict(N=2000, k=20, n=3, m=3, G=5, nq=30, D=6), 4, 7, 10),
    "ds1": (dict(N=1500, k=24, n=5, m=12, G=5, nq=20, D=12), 5, 9, 33),
    "n1": (dict(N=1500, k=24, n=1, m=4, G=5, nq=20, D=16), 5, 5, 10),
    # the graph degrees of the parameter study of Sec. 5 (n = 64, n = 128) with 16-byte codes
    "deep_n64": (dict(kind="deep", N=20000, k=200, n=64, m=16, G=32, nq=30), 8, 128, 50),
    "deep_n128": (dict(kind="deep", N=20000, k=300, n=128, m=16, G=32, nq=30), 6, 192, 50),
    "sift_n64_m16": (dict(N=20000, k=200, n=64, m=16, G=32, nq=30), 8, 128, 100),
    # data far from the origin: SIFT-like values + 1 000 per coordinate, DEEP-like + a constant vector
    "sift_shifted": (dict(N=20011, k=100, n=7, m=8, G=16, nq=77), 9, 25, 100, 1000.0),
    "deep_shifted": (dict(kind="deep", N=15000, k=96, n=8, m=16, G=32, nq=50), 8, 20, 50, 3.0),
    "sift_shifted_generic": (dict(N=3000, k=32, n=4, m=4, G=8, nq=40, D=32), 6, 10, 20, 1000.0),
}


@pytest.fixture(params=["stream", "generic"])
def scan_kind(request):
    """Every case runs twice: with the scan the shape selects (one table per query and a stored term
    per point where m is 8 or 16, several lists per wave when they are short), and with the
    per-cell / per-sub-region tables of Sec. 3.3.2 (2m lookups per point) forced."""
    return request.param


@pytest.mark.parametrize("name", list(CASES))
def test_build_encode_search_against_oracle(vlq, oracle_mod, name, scan_kind):
    kw, w1, w2, K, *rest = CASES[name]
    pr = shifted(problem(**kw), rest[0] if rest else 0.0)
    idx = make_index(vlq, pr)
    try:
        if scan_kind == "generic":
            vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SCAN_GENERIC, 1)
        Sg, Eg = gpu_graph(vlq, idx, pr)
        assert check_graph(oracle_mod, pr, Sg, Eg), "graph differs from the oracle's inside a tie band: pick another seed"
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc, soft = check_encode(oracle_mod, pr, S, E, pr.X, gpu_encode(vlq, idx, pr.X, pr.m))
        # search on the oracle's own index, loaded into the library
        load_oracle_index(vlq, idx, enc)
        assert vlq.vlq_index_ntotal(idx) == len(pr.X) and vlq.vlq_index_is_finalized(idx)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        # small codebooks: most graph edges are mutual, so mirrored-line ties at the cut are frequent
        # (such a query is still compared in full, for the GPU's choice among the tied lines)
        soft = 0.6 if pr.k < 30 else 0.25
        _, nsoft = check_search(oracle_mod, pr, S, E, lists, pr.Y, w1, w2, K, gpu_search(vlq, idx, pr.Y, w1, w2, K),
                                max_soft=soft)
        print(f"{name}/{scan_kind}: {nsoft} of {len(pr.Y)} queries compared for a tied choice of sub-regions")
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("qlam", [(0.0, 1.0), "grid"])
@pytest.mark.parametrize("name", ["sift_ragged", "deep_m16"])
def test_restricted_query_lambda(vlq, oracle_mod, name, qlam):
    """Region traversal with the query's lambda restricted to a range (Sec. 3.3.1 variant): the segment
    between the two centroids, and the part of the line the lambda byte can express.  Same protocol
    as above; the selection must really differ from the unrestricted one for some queries."""
    kw, w1, w2, K = CASES[name]
    pr = problem(**kw)
    if qlam == "grid":
        qlam = (oracle_mod.LAMBDA_LO, oracle_mod.LAMBDA_HI)
    idx = make_index(vlq, pr)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
        load_oracle_index(vlq, idx, enc)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        free = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        vlq.vlq_index_set_query_lambda_range(idx, *qlam)
        got = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        # a restricted lambda sits on the end of its range for many lines of a cell, and all lines of a cell
        # clamped to lambda = 0 score exactly its coarse distance: ties at the cut are common
        check_search(oracle_mod, pr, S, E, lists, pr.Y, w1, w2, K, got, qlam=qlam, max_soft=0.5)
        assert (np.sort(free[4], axis=1) != np.sort(got[4], axis=1)).any(1).mean() > 0.2
        with pytest.raises(vlq.VlqError):
            vlq.vlq_index_set_query_lambda_range(idx, 1.0, 0.0)
        # back to the whole line: the first results again
        vlq.vlq_index_set_query_lambda_range(idx, -np.inf, np.inf)
        again = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        for x, y in zip(free, again):
            assert np.array_equal(x, y)
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("lo,hi,n", [(-0.125, 0.5, 6), (-1.0, 0.5, 6), (0.0, 1e-20, 1)])
def test_other_lambda_grids(vlq, oracle_mod, lo, hi, n):
    """The byte grid of lambda is an index parameter: a finer grid, a wider one, and the
    degenerate grid whose 256 values are all (numerically) zero with one edge per cell, which
    turns the index into a plain inverted file with residuals to the cell centroid."""
    pr = problem(N=6000, k=48, n=n, m=8, G=12, nq=40)
    lo, hi = float(np.float32(lo)), float(np.float32(hi))  # the values the library receives
    idx = make_index(vlq, pr, lo=lo, hi=hi)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc, _ = check_encode(oracle_mod, pr, S, E, pr.X, gpu_encode(vlq, idx, pr.X, pr.m), grid=(lo, hi))
        if hi < 1e-10:  # every anchor is the centroid itself
            rec = oracle_mod.reconstruct(pr.C, S, pr.P, enc.cell, enc.edge, enc.lamq, enc.codes, lo, hi)
            rec0 = pr.C[enc.cell].astype(np.float64) + np.concatenate(
                [pr.P[p][enc.codes[:, p]] for p in range(pr.m)], axis=1).astype(np.float64)
            assert np.allclose(rec, rec0, rtol=0, atol=1e-12)
        load_oracle_index(vlq, idx, enc)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        w1 = 7
        w2 = 7 if n == 1 else 15
        check_search(oracle_mod, pr, S, E, lists, pr.Y, w1, w2, 30, gpu_search(vlq, idx, pr.Y, w1, w2, 30),
                     max_soft=0.3, grid=(lo, hi))
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("kind,fp32", [("sift", False), ("deep", False), ("sift", True)])
def test_encode_with_both_coarse_products(vlq, oracle_mod, kind, fp32):
    """Alg. 1 + 2 with the nearest-centroid shortlist from the split-bf16 product (integer-valued and
    real-valued data: without and with low halves) and from the fp32 product; several ragged tiles."""
    pr = problem(kind=kind, N=6000, k=300, n=6, m=8, G=16, nq=8)
    idx = make_index(vlq, pr)
    try:
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_COARSE_FP32, int(fp32))
        S, E = oracle_mod.graph(pr.C, pr.n)
        check_encode(oracle_mod, pr, S, E, pr.X, gpu_encode(vlq, idx, pr.X, pr.m))
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("dup,fp32", [(0, False), (600, False), (0, True)])
def test_cell_selection_with_many_centroids(vlq, oracle_mod, dup, fp32):
    """Alg. 3, first loop, at a codebook size where the cells come from the two sweeps of the bf16
    product (and, for comparison, from the fp32 distance matrix).  With `dup` coinciding centroids
    the candidate lists of the queries near them overflow and the exact ranking over all centroids
    takes over; ties go to the smaller index."""
    pr = problem(N=4000, k=1024, n=4, m=8, G=64, nq=300, D=32, iters=2)
    C = pr.C.copy()
    if dup:
        C[100:100 + dup] = C[100]
    pr2 = Problem(pr.kind, pr.X, pr.Y, C, pr.P, pr.n)
    Y = pr.Y.copy()
    if dup:
        Y[:20] = C[100] + np.arange(20, dtype=np.float32)[:, None]  # queries that see the whole tie
    idx = make_index(vlq, pr2, base=pr.X[:500])
    try:
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_COARSE_FP32, int(fp32))
        dist = oracle_mod.coarse(C, Y)
        for w1 in (1, 7, 32):
            # the whole batch, and a handful of queries (cells from rows of the fp32 distance matrix)
            for nqs in (len(Y), 24):
                od, oi, cells, cd, sub, ss = gpu_search(vlq, idx, Y[:nqs], w1, min(w1 * pr.n, 16), 10)
                for q in range(nqs):
                    check_selection(cells[q], dict(enumerate(dist[q])), w1, what=f"w1 {w1} query {q} of {nqs} cells")
                    assert np.allclose(cd[q], dist[q][cells[q]], rtol=DTOL, atol=1e-3)
                if dup:
                    ref = oracle_mod.select_smallest(dist[:20], w1)
                    assert (cells[:20] == ref).all()  # exact ties are ordered by index
        if dup:
            # hundreds of exactly equal line scores (the probed cells coincide, their edges have length
            # zero, so every score is the cell distance): the cut is taken by label
            w1, w2 = 100, 300
            od, oi, cells, cd, sub, ss = gpu_search(vlq, idx, Y[:20], w1, w2, 10)
            Sg, Eg = gpu_graph(vlq, idx, pr2)
            score, label = oracle_mod.subregion_scores(dist[:20], Sg, Eg.astype(np.float64), cells)
            pick = oracle_mod.select_smallest(score, w2, key=label)
            for q in range(20):
                assert (cells[q] == oracle_mod.select_smallest(dist[q:q + 1], w1)[0]).all()
                want = pick[q]  # with a key the oracle returns the keys (labels) of the selection
                assert sorted(sub[q].tolist()) == sorted(want.tolist()), f"query {q}: sub-regions at an exact tie"
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("fp32", [False, True])
def test_encode_with_coinciding_centroids(vlq, oracle_mod, fp32):
    """Alg. 1 where hundreds of centroids coincide: the nearest-centroid shortlist of the vectors near
    them holds more columns inside the rounding band than it has room for, is handed on as incomplete
    and those vectors are ranked exactly over all centroids.  Exactly equal distances go to the
    smaller index (Eq. 2), all lines of the chosen cell have length zero (edge 0, lambda 0): cell,
    edge and byte must equal the oracle's, not merely lie in its tie band."""
    pr = problem(N=4000, k=1024, n=4, m=8, G=64, nq=8, D=32, iters=2)
    C = pr.C.copy()
    C[100:700] = C[100]
    C[900:905] = C[900]  # a handful only: fits the shortlist, still an exact tie
    rng = np.random.default_rng(4)
    X = pr.X.copy()
    X[:300] = C[100] + rng.normal(scale=2.0, size=(300, pr.D)).astype(np.float32)
    X[300:400] = C[900] + rng.normal(scale=2.0, size=(100, pr.D)).astype(np.float32)
    pr2 = Problem(pr.kind, X, pr.Y, C, pr.P, pr.n)
    idx = make_index(vlq, pr2)
    try:
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_COARSE_FP32, int(fp32))
        S, E = oracle_mod.graph(C, pr.n)
        got = gpu_encode(vlq, idx, X, pr.m)
        enc, _ = check_encode(oracle_mod, pr2, S, E, X, got, max_soft=1.0)
        near = np.concatenate([np.nonzero(enc.cell == 100)[0], np.nonzero(enc.cell == 900)[0]])
        assert len(near) >= 380
        assert (got[0][near] == enc.cell[near]).all() and (got[1][near] == enc.edge[near]).all()
        assert (got[1][near] == 0).all() and (got[2][near] == 85).all()
        assert (got[3][near] == enc.codes[near]).mean() > 0.99
        # the same through the Lloyd assignment (nearest centroid only)
        a = torch.empty(len(X), dtype=torch.int32, device=DEV)
        vlq.vlq_kmeans(dev(X), len(X), pr.D, pr.k, 0, dev(C), a, None)
        torch.cuda.synchronize()
        assert (a.cpu().numpy()[near] == enc.cell[near]).all()
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("dup", [0, 600, 1500])
def test_cell_selection_with_long_column_splits(vlq, oracle_mod, dup):
    """A batch and a codebook large enough that each column split of the first sweep spans eight tiles
    or more: the sweep then bounds the w1-th smallest distance from every other tile only, and the
    second sweep lists about twice as many columns for the exact ranking.  Same checks as above on a
    sample of the queries; with coinciding centroids the lists of the queries near them overflow."""
    pr = problem(N=2000, k=8192, n=2, m=8, G=256, nq=8192, D=32, iters=1)
    C = pr.C.copy()
    Y = pr.Y.copy()
    if dup:
        C[100:100 + dup] = C[100]
        Y[:20] = C[100] + np.arange(20, dtype=np.float32)[:, None]
    pr2 = Problem(pr.kind, pr.X, Y, C, pr.P, pr.n)
    idx = make_index(vlq, pr2, base=pr.X[:500])
    try:
        rng = np.random.default_rng(5)
        qs = np.concatenate([np.arange(20), rng.choice(len(Y), 180, replace=False)])
        dist = oracle_mod.coarse(C, Y[qs])
        for w1 in (16, 64):
            od, oi, cells, cd, sub, ss = gpu_search(vlq, idx, Y, w1, 2 * w1, 10)
            assert (cells >= 0).all() and (np.sort(cells, axis=1)[:, 1:] != np.sort(cells, axis=1)[:, :-1]).all()
            for r, q in enumerate(qs):
                check_selection(cells[q], dict(enumerate(dist[r])), w1, what=f"w1 {w1} query {q} cells")
                assert np.allclose(cd[q], dist[r][cells[q]], rtol=DTOL, atol=1e-3)
            if dup:
                assert (cells[:20] == oracle_mod.select_smallest(dist[:20], w1)).all()
            # a handful of queries at this codebook size: exact distances to all centroids, cells straight from
            # them (with 1500 coinciding centroids by repeated selection over the whole row)
            od, oi, cells, cd, sub, ss = gpu_search(vlq, idx, Y[:20], w1, 2 * w1, 10)
            for q in range(20):
                check_selection(cells[q], dict(enumerate(dist[q])), w1, what=f"w1 {w1} query {q} of 20 cells")
                assert np.allclose(cd[q], dist[q][cells[q]], rtol=DTOL, atol=1e-3)
            if dup:
                assert (cells == oracle_mod.select_smallest(dist[:20], w1)).all()
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("split", [0, 1])
def test_cell_selection_when_the_bf16_parts_mislead(vlq, oracle_mod, split):
    """Alg. 3, first loop, on centroids built against the sweeps' arithmetic: every component sits a hair below or
    above a bf16 rounding boundary, so the hi parts of two kinds of centroids differ by 2^-7 of each component
    while the centroids themselves differ by 2^-19, and the approximate distances order the kinds, not the
    centroids.  The error band of the sweeps has to take in nearly every column and hand the decision to the
    exact ranking: the cells must be the oracle's (ties inside the fp32 resolution of the exact sums aside)."""
    rng = np.random.default_rng(17)
    D, k, nq, w1 = 32, 4096, 96, 8
    pr = problem(N=2000, k=64, n=2, m=8, G=16, nq=8, D=D, iters=1)  # (for the PQ codebooks and base vectors only)
    base = (rng.choice([-1.0, 1.0], size=D) * 2.0 ** rng.integers(-1, 2, size=D)).astype(np.float64)
    kind = rng.integers(0, 2, size=(k, 1)) * 2 - 1                      # -1: rounds down, +1: rounds up
    delta = rng.integers(-2, 3, size=(k, D))
    C = (base * (1.0 + 2.0 ** -8 + kind * 2.0 ** -20 + delta * 2.0 ** -23)).astype(np.float32)
    Y = (base * (0.9 + rng.integers(-64, 65, size=(nq, D)) * 2.0 ** -10)).astype(np.float32)
    pr2 = Problem(pr.kind, pr.X, Y, C, pr.P, 2)
    idx = make_index(vlq, pr2, base=pr.X[:500])
    try:
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_COARSE_SPLIT, split)
        dist = oracle_mod.coarse(C, Y)
        od, oi, cells, cd, sub, ss = gpu_search(vlq, idx, Y, w1, 2 * w1, 10)
        for q in range(nq):
            check_selection(cells[q], dict(enumerate(dist[q])), w1, what=f"query {q} cells")
            assert np.allclose(cd[q], dist[q][cells[q]], rtol=DTOL, atol=1e-6)
        # the kinds really are what the hi parts see: without the band the sweeps would pick by kind
        hi = (C.view(np.uint32) + 0x7FFF + ((C.view(np.uint32) >> 16) & 1)) >> 16 << 16
        assert len(np.unique(hi.view(np.float32)[:, 0])) == 2
    finally:
        vlq.vlq_index_free(idx)


def test_neighbour_distances_by_cell_and_by_query_agree(vlq):
    """The distances to the neighbour centroids (Alg. 3, second loop) computed cell by cell over the
    batch and computed inside the per-query kernel are the same sums: every output is identical.
    (The parity cases above run the cell-by-cell form; this pins the other one to it.)"""
    kw, w1, w2, K = CASES["sift_ragged"]
    pr = problem(**kw)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        a = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_NEIGHBOURS_PER_QUERY, 1)
        b = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("name", ["sift_ragged", "deep_m16"])
def test_batch_parts_and_small_batch_forms_agree(vlq, name):
    """A batch cut into parts whose region traversal runs on the index's second stream beside the scan of
    the part before (VLQ_OPT_PIPELINE_PARTS), and the forms a handful of queries take (exact or fp32-product
    distance matrix, ungrouped edge products: VLQ_OPT_SMALL_BATCH) against the ordinary ones, and the
    cell selection's sweeps over split operands (VLQ_OPT_COARSE_SPLIT) against the hi parts alone: every output
    identical."""
    kw, w1, w2, K = CASES[name]
    pr = problem(**kw)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        ref = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        for parts in (2, 4, 8):
            vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_PIPELINE_PARTS, parts)
            for rep in range(2):  # the second call reuses the events of the first
                got = gpu_search(vlq, idx, pr.Y, w1, w2, K)
                for x, y in zip(ref, got):
                    assert np.array_equal(x, y), f"{parts} parts"
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_PIPELINE_PARTS, 0)
        with pytest.raises(vlq.VlqError):
            vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_PIPELINE_PARTS, 99)
        Y = pr.Y[:20]
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SMALL_BATCH, 0)
        a = gpu_search(vlq, idx, Y, w1, w2, K)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SMALL_BATCH, 4096)
        b = gpu_search(vlq, idx, Y, w1, w2, K)
        assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2]) and np.array_equal(a[4], b[4])
        assert np.allclose(a[0], b[0], rtol=1e-6) and np.allclose(a[3], b[3], rtol=1e-6)
        # the two sweeps of the cell selection with split operands instead of the hi parts alone: the candidate
        # lists differ, the exact ranking of them does not
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SMALL_BATCH, 64)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_COARSE_SPLIT, 1)
        got = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        for x, y in zip(ref, got):
            assert np.array_equal(x, y), "split operands"
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("name", ["sift_ragged", "deep_m16", "small_d32"])
def test_both_encode_kernels_agree(vlq, oracle_mod, name):
    """Encoding has a kernel for the common shapes (a lane per vector in the product-quantisation step,
    four neighbour rows per pass in the line step) and a general one (a wave per vector).  The parity
    cases above run whichever serves their shape; here both run on the same vectors.  The line
    distances are summed in a different order, so an edge or a lambda byte may differ where the oracle
    sees a tie; everything else is identical, and each kernel passes the oracle check on its own."""
    kw = CASES[name][0]
    pr = problem(**kw)
    idx = make_index(vlq, pr)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_ENCODE_WAVE, 0)
        a = gpu_encode(vlq, idx, pr.X, pr.m)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_ENCODE_WAVE, 1)
        b = gpu_encode(vlq, idx, pr.X, pr.m)
        check_encode(oracle_mod, pr, S, E, pr.X, a)
        check_encode(oracle_mod, pr, S, E, pr.X, b)
        assert np.array_equal(a[0], b[0])
        same = (a[1] == b[1]) & (a[2] == b[2])
        assert same.mean() > 0.999
        assert np.array_equal(a[3][same], b[3][same])
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("name", ["sift_ragged", "deep_m16"])
def test_packed_and_per_list_scan_agree(vlq, name):
    """The streaming scan in its two forms - several short lists laid end to end over the lanes of a
    wave, or one list at a time - computes the same keys: every output is identical.  (Indexes with
    fewer than 64 points per list take the packed form by default, so the parity cases above run it;
    this pins the other form to it, at m = 8 and m = 16.)"""
    kw, w1, w2, K = CASES[name]
    pr = problem(**kw)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SCAN_PACKED, 1)
        a = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SCAN_PACKED, 0)
        b = gpu_search(vlq, idx, pr.Y, w1, w2, K)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
        # a single query is split over several workgroups in both forms
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SCAN_PACKED, 1)
        a = gpu_search(vlq, idx, pr.Y[:1], w1, w2, K)
        vlq.vlq_index_set_option(idx, vlq.VLQ_OPT_SCAN_PACKED, 0)
        b = gpu_search(vlq, idx, pr.Y[:1], w1, w2, K)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    finally:
        vlq.vlq_index_free(idx)


def test_largest_supported_shapes(vlq, oracle_mod):
    """The limits of include/vlq.h together: D = 1 024, m = 64, w1 = 512, w1 * n = 8 192 sub-regions ranked,
    w2 = 2 048 visited, K = 1 024 (fp32 coarse product, generic scan)."""
    pr = problem(N=4000, k=520, n=16, m=64, G=12, nq=4, D=1024, iters=2)
    idx = make_index(vlq, pr)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc, _ = check_encode(oracle_mod, pr, S, E, pr.X, gpu_encode(vlq, idx, pr.X, pr.m))
        load_oracle_index(vlq, idx, enc)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        w1, w2, K = 512, 2048, 1024
        check_search(oracle_mod, pr, S, E, lists, pr.Y, w1, w2, K, gpu_search(vlq, idx, pr.Y, w1, w2, K), max_soft=1.0)
    finally:
        vlq.vlq_index_free(idx)


def test_search_can_be_captured_in_a_graph(vlq):
    """After one call has sized the scratch memory, vlq_search only launches kernels on the given
    stream: it can be captured in a HIP graph.  Every replay (with new queries written into the
    captured input buffer, and ordinary work and synchronisations between replays) gives the rows
    of a plain call."""
    pr = problem(kind="deep", N=15000, k=96, n=8, m=16, G=32, nq=50)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        nq, w1, w2, K = 50, 8, 20, 50
        rng = np.random.default_rng(9)
        Yin = dev(pr.Y.copy())
        od = torch.empty(nq, K, device=DEV)
        oi = torch.empty(nq, K, dtype=torch.int32, device=DEV)
        vlq.vlq_search(idx, Yin, nq, w1, w2, K, od, oi)  # sizes the scratch
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            vlq.vlq_search(idx, Yin, nq, w1, w2, K, od, oi)
        for rep in range(4):
            Y = pr.Y[rng.permutation(nq)] + rng.normal(scale=0.01, size=pr.Y.shape).astype(np.float32)
            Yin.copy_(dev(Y))
            graph.replay()
            torch.cuda.synchronize()
            got_d, got_i = od.clone(), oi.clone()
            od2 = torch.empty(nq, K, device=DEV)
            oi2 = torch.empty(nq, K, dtype=torch.int32, device=DEV)
            vlq.vlq_search(idx, dev(Y), nq, w1, w2, K, od2, oi2)
            torch.cuda.synchronize()
            assert torch.equal(got_i, oi2) and torch.equal(got_d, od2), f"replay {rep}"
    finally:
        vlq.vlq_index_free(idx)


def test_large_batches_are_tiled_without_changing_results(vlq):
    """More queries than one internal tile (32 768): the same rows as when the queries are sent in
    pieces (a query's result does not depend on its batch)."""
    pr = problem(N=3000, k=32, n=4, m=8, G=8, nq=40, D=32)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        rng = np.random.default_rng(3)
        nq = 70001
        Y = pr.Y[rng.integers(0, len(pr.Y), nq)] + rng.normal(scale=0.5, size=(nq, pr.D)).astype(np.float32)
        Yd = dev(Y)
        od = torch.empty(nq, 10, device=DEV)
        oi = torch.empty(nq, 10, dtype=torch.int32, device=DEV)
        vlq.vlq_search(idx, Yd, nq, 4, 6, 10, od, oi)
        torch.cuda.synchronize()
        for lo, hi in [(0, 5), (32760, 32780), (65530, 65545), (69990, 70001)]:
            od2 = torch.empty(hi - lo, 10, device=DEV)
            oi2 = torch.empty(hi - lo, 10, dtype=torch.int32, device=DEV)
            vlq.vlq_search(idx, Yd[lo:hi].contiguous(), hi - lo, 4, 6, 10, od2, oi2)
            torch.cuda.synchronize()
            assert torch.equal(oi[lo:hi], oi2) and torch.equal(od[lo:hi], od2)
    finally:
        vlq.vlq_index_free(idx)


def test_lists_layout_matches_oracle(vlq, oracle_mod):
    """vlq_index_add + finalize: the four list arrays of Sec. 4, ids ascending inside a list."""
    pr = problem(N=20011, k=100, n=7, m=8, G=16, nq=77)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        nl = pr.k * pr.n
        off = torch.empty(nl + 1, dtype=torch.int64, device=DEV)
        ids = torch.empty(len(pr.X), dtype=torch.int32, device=DEV)
        codes = torch.empty(len(pr.X), pr.m, dtype=torch.uint8, device=DEV)
        lam = torch.empty(len(pr.X), dtype=torch.uint8, device=DEV)
        vlq.vlq_index_get_lists(idx, off, ids, codes, lam)
        torch.cuda.synchronize()
        off, ids, codes, lam = off.cpu().numpy(), ids.cpu().numpy(), codes.cpu().numpy(), lam.cpu().numpy()
        got = gpu_encode(vlq, idx, pr.X, pr.m)
        want = oracle_mod.make_lists(pr.k, pr.n, got[0], got[1], got[2], got[3])  # layout only: same fields
        assert (off == want.off).all() and (ids == want.ids).all()
        assert (codes == want.codes).all() and (lam == want.lamq).all()
        assert sorted(ids.tolist()) == list(range(len(pr.X)))
    finally:
        vlq.vlq_index_free(idx)


def test_tiny_config_end_to_end(vlq, oracle_mod):
    """The small SIFT-like configuration: N = 100000, D = 128, k = 256, n = 8, m = 8,
    w1 = 8, 32 sub-regions, K = 100; search parity on every query, encode parity on
    every point, recall equal to the oracle's."""
    pr = problem(N=100000, nq=1000, k=256, n=8, m=8, G=64, iters=10, seed=0, ntrain=20000)
    idx = make_index(vlq, pr)
    try:
        Sg, Eg = gpu_graph(vlq, idx, pr)
        assert check_graph(oracle_mod, pr, Sg, Eg)
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc, soft = check_encode(oracle_mod, pr, S, E, pr.X, gpu_encode(vlq, idx, pr.X, pr.m), max_soft=0.002)
        load_oracle_index(vlq, idx, enc)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        got = gpu_search(vlq, idx, pr.Y, 8, 32, 100)
        # about 3 % of the queries have a mirrored pair of lines straddling the cut at w2 = 32
        tr, soft = check_search(oracle_mod, pr, S, E, lists, pr.Y, 8, 32, 100, got, max_soft=0.06)
        assert (got[1] == tr.out_id[:, :100]).mean() > 0.95
        from parity import STATS
        print("parity stats so far:", STATS)
    finally:
        vlq.vlq_index_free(idx)


def test_small_batches_use_split_scan(vlq, oracle_mod):
    """nq = 1, 2, 5: each query is split over several workgroups and merged."""
    pr = problem(N=20011, k=100, n=7, m=8, G=16, nq=77)
    idx = make_index(vlq, pr)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
        load_oracle_index(vlq, idx, enc)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes)
        for nq, K in ((1, 100), (2, 1), (5, 10), (3, 1024)):
            Y = pr.Y[10 : 10 + nq]
            check_search(oracle_mod, pr, S, E, lists, Y, 12, 40, K, gpu_search(vlq, idx, Y, 12, 40, K))
    finally:
        vlq.vlq_index_free(idx)


def test_edge_cases(vlq, oracle_mod):
    pr = problem(N=3000, k=32, n=4, m=8, G=8, nq=40, D=32)
    idx = make_index(vlq, pr)
    try:
        # empty index: every row padded
        od, oi, *_ = gpu_search(vlq, idx, pr.Y, 4, 6, 7)
        assert np.isinf(od).all() and (oi == -1).all()
        # nq = 0 and nb = 0 are no-ops
        vlq.vlq_search(idx, dev(pr.Y), 0, 4, 6, 7, torch.empty(1, device=DEV), torch.empty(1, dtype=torch.int32, device=DEV))
        vlq.vlq_index_add(idx, dev(pr.X), 0)
        # fewer candidates than K, custom ids, two add calls
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc = oracle_mod.encode(pr.C, S, E, pr.P, pr.X)
        ids = (np.arange(len(pr.X)) * 7 + 3).astype(np.int32)
        half = 1234
        for sl in (slice(0, half), slice(half, None)):
            vlq.vlq_index_add_encoded(idx, dev(enc.cell[sl]), dev(enc.edge[sl]), dev(enc.lamq[sl]), dev(enc.codes[sl]),
                                      dev(ids[sl]), len(enc.cell[sl]))
        assert not vlq.vlq_index_is_finalized(idx)
        with pytest.raises(vlq.VlqError):
            gpu_search(vlq, idx, pr.Y, 4, 6, 7)
        vlq.vlq_index_finalize(idx)
        lists = oracle_mod.make_lists(pr.k, pr.n, enc.cell, enc.edge, enc.lamq, enc.codes, ids)
        check_search(oracle_mod, pr, S, E, lists, pr.Y, 1, 1, 400, gpu_search(vlq, idx, pr.Y, 1, 1, 400))
        # exhaustive probe
        check_search(oracle_mod, pr, S, E, lists, pr.Y, pr.k, pr.k * pr.n, 50, gpu_search(vlq, idx, pr.Y, pr.k, pr.k * pr.n, 50))
        # argument errors
        for bad in ((0, 1, 1), (pr.k + 1, 1, 1), (4, 17, 1), (4, 0, 1), (4, 6, 0), (4, 6, 5000)):
            with pytest.raises(vlq.VlqError) as ei:
                gpu_search(vlq, idx, pr.Y, *bad)
            assert ei.value.code == vlq.VLQ_EINVAL
        with pytest.raises(vlq.VlqError):
            bad_cell = enc.cell[:10].copy()
            bad_cell[3] = pr.k
            vlq.vlq_index_add_encoded(idx, dev(bad_cell), dev(enc.edge[:10]), dev(enc.lamq[:10]), dev(enc.codes[:10]), None, 10)
    finally:
        vlq.vlq_index_free(idx)


@pytest.mark.parametrize("copies", [5000, 20000])
def test_degenerate_data(vlq, oracle_mod, copies):
    """All base vectors identical: one long list (sorted by id in the second / third tier of the
    per-list sort), every distance tied, order by id."""
    pr = problem(N=3000, k=32, n=4, m=8, G=8, nq=40, D=32)
    X = np.repeat(pr.X[:1], copies, axis=0)
    idx = make_index(vlq, pr, base=X)
    try:
        S, E = oracle_mod.graph(pr.C, pr.n)
        enc = oracle_mod.encode(pr.C, S, E, pr.P, X[:1])
        cell, edge, lamq, codes = gpu_encode(vlq, idx, X, pr.m)
        assert (cell == enc.cell[0]).all() and (edge == enc.edge[0]).all()
        assert (lamq == enc.lamq[0]).all() and (codes == enc.codes[0]).all()
        Y = np.concatenate([X[:1], pr.Y[:3]])
        od, oi, *_ = gpu_search(vlq, idx, Y, pr.k, pr.k * pr.n, 64)
        assert (oi == np.arange(64)[None, :]).all()
        assert (od == od[:, :1]).all()
    finally:
        vlq.vlq_index_free(idx)


def test_profile_hooks(vlq):
    pr = problem(N=3000, k=32, n=4, m=8, G=8, nq=40, D=32)
    idx = make_index(vlq, pr, base=pr.X)
    try:
        vlq.vlq_profile_enable(idx, True)
        gpu_search(vlq, idx, pr.Y, 4, 6, 7)
        prof = vlq.vlq_profile_read(idx)
        assert prof["scan"][1] == 2 and prof["scan"][0] > 0 and prof["coarse"][1] == 2
        vlq.vlq_profile_enable(idx, False)
        gpu_search(vlq, idx, pr.Y, 4, 6, 7)
        assert vlq.vlq_profile_read(idx)["scan"][1] == 0
    finally:
        vlq.vlq_index_free(idx)
