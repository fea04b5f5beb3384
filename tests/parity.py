"""Comparison of GPU results with the fp64 oracle.

Integer outputs must be identical wherever the oracle's gap between the chosen
alternative and the best rejected one exceeds GAP (1e-5, relative to the scale
stated per decision); inside that band the GPU's choice must be one of the
near-tied alternatives.  Floating-point outputs must agree to DTOL relative.
The lambda byte must be equal, or one step apart when the oracle's grid
coordinate lies within LAM_WINDOW of a half-integer.

Two bands carry a term that is absolute, each with its derivation:

  * Returned distances.  The scan does not rebuild the point: it sums the terms of
    Eq. 16-17 (the stored per-point term, m table entries, a, lambda (b - a)), each
    of which can be far larger than the distance.  Every term is rounded once and so
    is every partial sum: at most abs_terms(m) = m + 4 roundings, each of at most
    2^-24 of the size of the terms.  `term_scale` bounds that size from the inputs:
    the largest coarse distance of the probed cells, plus what the inner products
    with the codewords can reach relative to the mean of the centroids (both the
    stored term and the table are taken relative to it, so the bound does not move
    when data, queries and centroids are translated together).
  * Codes.  The residual of Eq. 12 is formed in fp64 and rounded once to fp32, which
    moves it by at most 2^-24 of its own norm; the distance to a codeword moves by
    no more than the residual does.  Two codewords whose distances (not squared)
    differ by less than RES_ROUNDINGS of those roundings are a tie (both distances,
    factor 2 margin).  This matters where sub-spaces have one or two dimensions and
    256 codewords sit closer together than the rounding of the residual.
"""
from __future__ import annotations

import numpy as np

GAP = 1e-5
DTOL = 1e-4
EPS32 = 2.0 ** -24
LAM_WINDOW = 2e-3  # of a grid step, around the half-integers
RES_ROUNDINGS = 4


def abs_terms(m):
    return m + 4


def term_scale(a_max, y, Cb, P):
    """Bound on the size of the terms a returned distance is summed from (see above), for one
    query y: a_max + R^2 + 2 R (2 |y - mu| + sqrt(a_max)), R the largest norm a concatenation of
    codewords can have, mu the mean of the centroids."""
    mu = np.asarray(Cb, np.float64).mean(0)
    R = np.sqrt(sum((np.asarray(P[p], np.float64) ** 2).sum(1).max() for p in range(len(P))))
    ym = np.linalg.norm(np.asarray(y, np.float64) - mu)
    return a_max + R * R + 2.0 * R * (2.0 * ym + np.sqrt(a_max))


def check_selection(got, val_of, w, scale=None, what=""):
    """`got`: sequence of w labels chosen by the GPU (ascending by value, ties by
    label).  `val_of`: dict label -> oracle value for every eligible label.
    Returns True if the chosen SET equals the oracle's (the order may differ
    inside the tie band: mirrored lines l(c_i,c_j) / l(c_j,c_i) tie exactly in
    exact arithmetic), False if the set differs only inside the tie band;
    raises AssertionError otherwise."""
    items = sorted((v, l) for l, v in val_of.items())
    want = [l for _, l in items[:w]]
    got = [int(g) for g in got]
    if got == want:
        return True
    assert len(set(got)) == len(got), f"{what}: duplicate labels"
    assert len(got) == min(w, len(items)) or got[len(items):] == [-1] * (w - len(items)), f"{what}: wrong count"
    got = got[: len(items)]
    cut = items[min(w, len(items)) - 1][0]
    tol = GAP * (abs(cut) if scale is None else scale)
    for l in got:
        assert l in val_of, f"{what}: label {l} is not eligible"
        assert val_of[l] <= cut + tol, f"{what}: label {l} value {val_of[l]} beyond cut {cut}"
    sure = {l for v, l in items if v < cut - tol}
    assert sure <= set(got), f"{what}: missing labels {sorted(sure - set(got))[:5]}"
    vals = [val_of[l] for l in got]
    for a, b in zip(vals, vals[1:]):
        assert a <= b + tol, f"{what}: order violated beyond the tie band"
    return set(got) == set(want)


def reconciled_graph(oracle, Cb, n, rows, S_gpu):
    """Oracle graph rows (S, E as oracle.sparse_graph gives them) for the given centroids, made
    consistent with the library's numbering of the edges: two neighbours whose distances from c_i
    agree to fp32 resolution are ordered by index on the GPU and by their fp64 distances in the
    oracle, and an edge label i * n + j then names different lines on the two sides.  Such a row
    must equal the oracle's up to the tie band (checked here); the library's order is then adopted,
    with the squared edge lengths of that order in fp64, so that everything downstream is compared
    for the library's (valid) choice.  Returns (S, E, number of rows adopted)."""
    S, E = oracle.sparse_graph(Cb, n, rows)
    Cd = None
    adopted = 0
    for i in np.unique(np.asarray(rows)):
        if (S_gpu[i] == S[i]).all():
            continue
        if Cd is None:
            Cd = np.asarray(Cb, np.float64)
        d = ((Cd - Cd[i]) ** 2).sum(1)
        val = {int(j): float(d[j]) for j in np.argsort(d)[: 4 * n + 4] if j != i}
        check_selection(S_gpu[i], val, n, what=f"graph row {i}")
        S[i] = S_gpu[i]
        E[i] = d[S_gpu[i]]
        adopted += 1
    return S, E, adopted


STATS = {"max_abs_over_eps_scale": 0.0, "max_rel": 0.0}


def check_topk(g_d, g_i, o_d, o_i, K, what="", scale=0.0, m=8):
    """Final results of one query: GPU (g_d, g_i)[K] against the oracle's first
    K' >= K results (o_d, o_i).  `scale`: term_scale of the query, m the number of
    code bytes.  Returns True when the id sets are identical."""
    abs_tol = abs_terms(m) * EPS32 * scale
    o_map = {int(i): float(d) for d, i in zip(o_d, o_i) if i >= 0}
    n_valid = min(K, len(o_map))
    exact = True
    for r in range(K):
        gi, gd = int(g_i[r]), float(g_d[r])
        if r >= n_valid:
            assert gi == -1 and np.isinf(gd), f"{what}: row not padded at {r}"
            continue
        assert gi in o_map, f"{what}: id {gi} at rank {r} is not among the oracle's best {len(o_map)}"
        od = o_map[gi]
        assert abs(gd - od) <= DTOL * max(od, 1e-30) + abs_tol, f"{what}: distance {gd} vs {od} at rank {r}"
        if scale > 0:
            STATS["max_abs_over_eps_scale"] = max(STATS["max_abs_over_eps_scale"], abs(gd - od) / (EPS32 * scale))
        STATS["max_rel"] = max(STATS["max_rel"], abs(gd - od) / max(od, 1e-30))
        if gi != int(o_i[r]):
            exact = False
            ref = float(o_d[r])
            assert abs(od - ref) <= GAP * max(ref, 1e-30) + abs_tol, f"{what}: id {gi} at rank {r} differs beyond the tie band"
    assert len({int(i) for i in g_i if i >= 0}) == n_valid, f"{what}: duplicate ids"
    return {int(i) for i in g_i[:n_valid]} == {int(i) for i in o_i[:n_valid]}
