"""CPU oracle of the VLQ-ADC build and query definitions (test infrastructure).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It wraps ``vlq_oracle.c`` (plain C,
fp64, definition-level) with ctypes; the wrappers only marshal numpy arrays.
The product library never loads it and the two share no code.

Sections / equations cited are those of the paper: Eq. 2 (VQ), Eq. 7-8 (line
distance and lambda), Eq. 12-13 (residual), Alg. 1-3, Eq. 14 (ADC distance).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vlq_oracle.c")
_SO = os.path.join(_HERE, "libvlq_oracle.so")

LAMBDA_LO = -0.25
LAMBDA_HI = 0.5


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (about a second)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        )
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.vlqo_lambda_dequant.restype = C.c_double
        _lib.vlqo_lambda_dequant.argtypes = [C.c_int, C.c_double, C.c_double]
        _lib.vlqo_lambda_coord.restype = C.c_double
        _lib.vlqo_lambda_coord.argtypes = [C.c_double, C.c_double, C.c_double]
        _lib.vlqo_lambda_quant.restype = C.c_int
        _lib.vlqo_lambda_quant.argtypes = [C.c_double, C.c_double, C.c_double]
        _lib.vlqo_line_lambda.restype = C.c_double
        _lib.vlqo_line_lambda.argtypes = [C.c_double] * 3
        _lib.vlqo_line_dist2.restype = C.c_double
        _lib.vlqo_line_dist2.argtypes = [C.c_double] * 4
        _lib.vlqo_num_threads.restype = C.c_int
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().vlqo_num_threads())


def set_num_threads(t: int) -> None:
    lib().vlqo_set_num_threads(C.c_int(int(t)))


# ---- scalar pieces (Eq. 7, Eq. 8, lambda byte) ---------------------------


def line_lambda(a, b, c) -> float:
    return float(lib().vlqo_line_lambda(float(a), float(b), float(c)))


def line_dist2(a, b, c, lam) -> float:
    return float(lib().vlqo_line_dist2(float(a), float(b), float(c), float(lam)))


def lambda_quant(lam, lo=LAMBDA_LO, hi=LAMBDA_HI) -> int:
    return int(lib().vlqo_lambda_quant(float(lam), float(lo), float(hi)))


def lambda_dequant(q, lo=LAMBDA_LO, hi=LAMBDA_HI) -> float:
    return float(lib().vlqo_lambda_dequant(int(q), float(lo), float(hi)))


def lambda_coord(lam, lo=LAMBDA_LO, hi=LAMBDA_HI) -> float:
    return float(lib().vlqo_lambda_coord(float(lam), float(lo), float(hi)))


# ---- graph ---------------------------------------------------------------


def graph(Cb, n, rows=None):
    """n-NN graph rows (Sec. 3.1): (S int32 [r x n], E float64 [r x n])."""
    Cb = _f32(Cb)
    k, D = Cb.shape
    if rows is None:
        nrows, rp = k, None
    else:
        rows = _i32(rows)
        nrows, rp = len(rows), _p(rows, C.c_int32)
    S = np.empty((nrows, n), np.int32)
    E = np.empty((nrows, n), np.float64)
    lib().vlqo_graph_rows(_p(Cb, C.c_float), k, D, n, rp, nrows, _p(S, C.c_int32), _p(E, C.c_double))
    return S, E


def sparse_graph(Cb, n, rows):
    """Full-shape (S, E) with only the given rows filled (others -1 / nan)."""
    Cb = _f32(Cb)
    k = Cb.shape[0]
    rows = np.unique(_i32(rows))
    S = np.full((k, n), -1, np.int32)
    E = np.full((k, n), np.nan, np.float64)
    s, e = graph(Cb, n, rows)
    S[rows] = s
    E[rows] = e
    return S, E


# ---- encoding ------------------------------------------------------------


@dataclass
class Encoded:
    cell: np.ndarray  # int32 [N]
    edge: np.ndarray  # int32 [N]
    lamq: np.ndarray  # uint8 [N]
    codes: np.ndarray  # uint8 [N x m]
    cell_d: np.ndarray  # float64 [N x 2] best / second-best VQ objective
    edge_d: np.ndarray  # float64 [N x 2] best / second-best line distance
    lam_coord: np.ndarray  # float64 [N] unrounded grid coordinate of lambda
    code_d: np.ndarray  # float64 [N x m x 2]


def vq_assign(Cb, X):
    Cb, X = _f32(Cb), _f32(X)
    k, D = Cb.shape
    N = X.shape[0]
    cell = np.empty(N, np.int32)
    cd = np.empty((N, 2), np.float64)
    lib().vlqo_vq_assign(_p(Cb, C.c_float), k, D, _p(X, C.c_float), C.c_int64(N), _p(cell, C.c_int32), _p(cd, C.c_double))
    return cell, cd


def lloyd_step(Cb, X):
    """One Lloyd iteration of k-means (the training of the codebooks, Sec. 2.1 / Sec. 5): rows
    of X go to their nearest centroid (Eq. 2, ties to the smaller index), every centroid with
    members becomes their mean (fp64), one without stays.  Returns (new centroids fp64,
    assignment, best / second-best objective per row)."""
    cell, cd = vq_assign(Cb, X)
    k, D = np.shape(Cb)
    new = np.array(Cb, np.float64)
    X64 = np.asarray(X, np.float64)
    for i in range(k):
        members = X64[cell == i]
        if len(members):
            new[i] = members.sum(0) / len(members)
    return new, cell, cd


def line_residual(Cb, S, X, cell, edge, lamq, lo=LAMBDA_LO, hi=LAMBDA_HI):
    """x - ((1 - l) c_i + l s_ij) with l the value of the lambda byte (Eq. 12), fp64."""
    Cb64 = np.asarray(Cb, np.float64)
    ci = Cb64[cell]
    sj = Cb64[np.asarray(S)[cell, edge]]
    lam = np.array([lambda_dequant(int(q), lo, hi) for q in lamq])[:, None]
    return np.asarray(X, np.float64) - ((1.0 - lam) * ci + lam * sj)


def encode(Cb, S, E, P, X, lo=LAMBDA_LO, hi=LAMBDA_HI) -> Encoded:
    """Alg. 1 + Alg. 2 for every row of X.  P: [m, 256, D/m]."""
    Cb, X, P = _f32(Cb), _f32(X), _f32(P)
    S = _i32(S)
    E = np.ascontiguousarray(E, np.float64)
    k, D = Cb.shape
    n = S.shape[1]
    m = P.shape[0]
    assert P.shape == (m, 256, D // m) and D % m == 0
    N = X.shape[0]
    out = Encoded(
        np.empty(N, np.int32), np.empty(N, np.int32), np.empty(N, np.uint8), np.empty((N, m), np.uint8),
        np.empty((N, 2)), np.empty((N, 2)), np.empty(N), np.empty((N, m, 2)),
    )
    lib().vlqo_encode(
        _p(Cb, C.c_float), k, D, n, _p(S, C.c_int32), _p(E, C.c_double), _p(P, C.c_float), m,
        C.c_double(lo), C.c_double(hi), _p(X, C.c_float), C.c_int64(N),
        _p(out.cell, C.c_int32), _p(out.edge, C.c_int32), _p(out.lamq, C.c_uint8), _p(out.codes, C.c_uint8),
        _p(out.cell_d, C.c_double), _p(out.edge_d, C.c_double), _p(out.lam_coord, C.c_double), _p(out.code_d, C.c_double),
    )
    return out


def reconstruct(Cb, S, P, cell, edge, lamq, codes, lo=LAMBDA_LO, hi=LAMBDA_HI):
    Cb, P = _f32(Cb), _f32(P)
    S = _i32(S)
    D = Cb.shape[1]
    n = S.shape[1]
    m = P.shape[0]
    cell, edge = _i32(cell), _i32(edge)
    lamq = np.ascontiguousarray(lamq, np.uint8)
    codes = np.ascontiguousarray(codes, np.uint8)
    N = cell.shape[0]
    Xh = np.empty((N, D), np.float64)
    lib().vlqo_reconstruct(
        _p(Cb, C.c_float), D, n, _p(S, C.c_int32), _p(P, C.c_float), m, C.c_double(lo), C.c_double(hi),
        _p(cell, C.c_int32), _p(edge, C.c_int32), _p(lamq, C.c_uint8), _p(codes, C.c_uint8), C.c_int64(N),
        _p(Xh, C.c_double),
    )
    return Xh


@dataclass
class Lists:
    """Inverted lists (Sec. 4): lengths as offsets, then ids / codes / lambda bytes,
    list l = cell * n + edge, ascending id inside a list."""

    off: np.ndarray  # int64 [k*n + 1]
    ids: np.ndarray  # int32 [N]
    codes: np.ndarray  # uint8 [N x m]
    lamq: np.ndarray  # uint8 [N]


def make_lists(k, n, cell, edge, lamq, codes, ids=None) -> Lists:
    N = len(cell)
    ids = np.arange(N, dtype=np.int32) if ids is None else _i32(ids)
    lab = cell.astype(np.int64) * n + edge.astype(np.int64)
    order = np.lexsort((ids, lab))
    cnt = np.bincount(lab, minlength=k * n)
    off = np.zeros(k * n + 1, np.int64)
    np.cumsum(cnt, out=off[1:])
    return Lists(off, np.ascontiguousarray(ids[order]), np.ascontiguousarray(codes[order]), np.ascontiguousarray(lamq[order]))


# ---- search, step by step (Alg. 3) ---------------------------------------


def coarse(Cb, Y):
    Cb, Y = _f32(Cb), _f32(Y)
    k, D = Cb.shape
    nq = Y.shape[0]
    dist = np.empty((nq, k), np.float64)
    lib().vlqo_coarse(_p(Cb, C.c_float), k, D, _p(Y, C.c_float), nq, _p(dist, C.c_double))
    return dist


def select_smallest(val, w, key=None):
    val = np.ascontiguousarray(val, np.float64)
    nq, ln = val.shape
    key = None if key is None else _i32(key)
    out = np.empty((nq, w), np.int32)
    lib().vlqo_select_smallest(_p(val, C.c_double), _p(key, C.c_int32), nq, ln, w, _p(out, C.c_int32))
    return out


def subregion_scores(dist, S, E, cells, qlam=(-np.inf, np.inf)):
    """Eq. 7-8 line scores of the w1 * n sub-regions of the probed cells; qlam = (lo, hi) restricts
    the query's lambda to that range before Eq. 7 is evaluated (default: the whole line)."""
    dist = np.ascontiguousarray(dist, np.float64)
    S = _i32(S)
    E = np.ascontiguousarray(E, np.float64)
    cells = _i32(cells)
    nq, k = dist.shape
    n = S.shape[1]
    w1 = cells.shape[1]
    score = np.empty((nq, w1 * n), np.float64)
    label = np.empty((nq, w1 * n), np.int32)
    lib().vlqo_subregion_scores(
        _p(dist, C.c_double), nq, k, n, _p(S, C.c_int32), _p(E, C.c_double), _p(cells, C.c_int32), w1,
        C.c_double(qlam[0]), C.c_double(qlam[1]), _p(score, C.c_double), _p(label, C.c_int32),
    )
    return score, label


def scan(Cb, S, P, lists: Lists, Y, sub, K, lo=LAMBDA_LO, hi=LAMBDA_HI):
    Cb, P, Y = _f32(Cb), _f32(P), _f32(Y)
    S = _i32(S)
    sub = _i32(sub)
    D = Cb.shape[1]
    n = S.shape[1]
    m = P.shape[0]
    nq, w2 = sub.shape
    out_d = np.empty((nq, K), np.float64)
    out_id = np.empty((nq, K), np.int32)
    ncand = np.empty(nq, np.int64)
    lib().vlqo_scan(
        _p(Cb, C.c_float), D, n, _p(S, C.c_int32), _p(P, C.c_float), m, C.c_double(lo), C.c_double(hi),
        _p(lists.off, C.c_int64), _p(lists.ids, C.c_int32), _p(lists.codes, C.c_uint8), _p(lists.lamq, C.c_uint8),
        _p(Y, C.c_float), nq, _p(sub, C.c_int32), w2, K, _p(out_d, C.c_double), _p(out_id, C.c_int32), _p(ncand, C.c_int64),
    )
    return out_d, out_id, ncand


@dataclass
class SearchTrace:
    dist: np.ndarray  # [nq x k] coarse distances
    cells: np.ndarray  # [nq x w1]
    score: np.ndarray  # [nq x w1*n] line scores in probed-cell order
    label: np.ndarray  # [nq x w1*n] list label of each score
    sub: np.ndarray  # [nq x w2] visited lists
    out_d: np.ndarray  # [nq x K]
    out_id: np.ndarray  # [nq x K]
    ncand: np.ndarray  # [nq]


def search(Cb, S, E, P, lists: Lists, Y, w1, w2, K, lo=LAMBDA_LO, hi=LAMBDA_HI, qlam=(-np.inf, np.inf)) -> SearchTrace:
    """Alg. 3 as the composition of its steps."""
    dist = coarse(Cb, Y)
    cells = select_smallest(dist, w1)
    score, label = subregion_scores(dist, S, E, cells, qlam)
    sub = select_smallest(score, w2, key=label)
    out_d, out_id, ncand = scan(Cb, S, P, lists, Y, sub, K, lo, hi)
    return SearchTrace(dist, cells, score, label, sub, out_d, out_id, ncand)


# ---- memory accounting (Sec. 3.1 and Sec. 5, memory paragraph) -----------


def graph_bytes(k, n) -> int:
    """indices + squared edge lengths of the n-NN graph."""
    return k * n * (4 + 4)

def second_level_vq_bytes(k, n, D) -> int:
    """what a VQ second level would store instead: k*n full-dimensional sub-centroids."""
    return k * n * D * 4

def index_bytes(N, k, n, D, m) -> int:
    """ids + codes + lambda bytes + codebook, graph and k x 256 x m table."""
    return 4 * N + m * N + N + 4 * k * (D + 2 * n + m * 256)
