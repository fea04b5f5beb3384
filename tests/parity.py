"""Comparison of GPU results with the fp64 oracle.

Integer outputs must be identical wherever the oracle's gap between the chosen
alternative and the best rejected one exceeds GAP (1e-5, relative to the scale
stated per decision); inside that band the GPU's choice must be one of the
near-tied alternatives.  Floating-point outputs must agree to DTOL relative.

Both bands are relative to the result.  Where fp32 arithmetic forms a small
result from much larger operands, the rounding of the operands is an absolute
error that no evaluation order in fp32 avoids, and the bands are widened by it:
  * Eq. 14 is evaluated as a sum of terms (Eq. 16-17) of the size of the
    query's distance to its probed cells, so a returned distance carries up to
    ABS_TERMS roundings of that size;
  * Eq. 8 gives lambda = (a + c - b) / 2c from three sums: where a and b are far
    larger than c (few centroids, points far from all of them) the difference
    cancels, and the grid coordinate of the lambda byte is uncertain by
    LAM_ROUNDINGS roundings of (a + b + c) / 2c grid steps (never less than the
    2e-3 of a step that well-conditioned lines need);
  * the residual of Eq. 12 is formed from a vector and an anchor of norm far
    above the spacing of the codewords when a sub-space has one dimension, so
    the distances to two codewords are each uncertain by RES_ROUNDINGS
    roundings of (|x^p| + |anchor^p|).
"""
from __future__ import annotations

import numpy as np

GAP = 1e-5
DTOL = 1e-4
EPS32 = 2.0 ** -24
ABS_TERMS = 32  # m + 4 additions of terms, each term itself a rounded sum, with margin
RES_ROUNDINGS = 16  # anchor (3 roundings) and subtraction (1), both codeword distances, factor 2 margin
LAM_ROUNDINGS = 32  # each of a, b, c: difference, square and a short accumulation tree per term, with margin


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


def check_topk(g_d, g_i, o_d, o_i, K, what="", scale=0.0):
    """Final results of one query: GPU (g_d, g_i)[K] against the oracle's first
    K' >= K results (o_d, o_i).  `scale`: the size of the terms the distance is
    summed from (the query's largest distance to a probed cell).  Returns True
    when the id sets are identical."""
    abs_tol = ABS_TERMS * EPS32 * scale
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
        if gi != int(o_i[r]):
            exact = False
            ref = float(o_d[r])
            assert abs(od - ref) <= GAP * max(ref, 1e-30) + abs_tol, f"{what}: id {gi} at rank {r} differs beyond the tie band"
    assert len({int(i) for i in g_i if i >= 0}) == n_valid, f"{what}: duplicate ids"
    return {int(i) for i in g_i[:n_valid]} == {int(i) for i in o_i[:n_valid]}
