"""Full-size checks, each in the launch configuration that bench.py times (10 000 queries, w1 = 64,
w2 = alpha w1 n, K = 100): mid SIFT-like (10^7 points, D = 128, k = 16 384, n = 32, m = 8), mid DEEP-like
(10^8, D = 96, k = 65 536, n = 32, m = 16), billion SIFT-like (10^9, D = 128, k = 65 536, n = 32, m = 8) and
billion DEEP-like (10^9, D = 96, k = 65 536, n = 64, m = 16).
The oracle cannot encode 10^7 points or more, so it is used on samples it can compute one by one; all of
its inputs come from the seeded generators (raw vectors are regenerated from the seed by id):

 * encoding of sampled base vectors (every field, tie-band protocol), and their place in the stored lists;
 * traversal (cells, sub-regions, scores) of sampled queries;
 * the whole top-K of the sampled queries (Alg. 3 second loop, Sec. 3.3.3): the lists the GPU visited are
   copied out of the library and scanned by the oracle (every point rebuilt, Eq. 14), and ids and
   distances are compared through the tie-band protocol of the small cases;
 * every returned (id, distance) of sampled queries once more from the raw data: the oracle encodes the
   raw vector of that id, rebuilds the approximated point and its distance to the query, and checks
   that the point's list was visited;
 * completeness probe: the exact nearest neighbour of a sampled query, if its list is visited and
   its ADC distance beats the K-th result, must be among the results;
 * batches of 1 to 3 000 of the same queries (which take the small- and medium-batch kernels) return the
   rows of the full batch bit for bit.
"""
import numpy as np
import pytest
import torch

import datagen
from datagen import workloads
from parity import DTOL, GAP, LAM_WINDOW, check_selection, check_topk, reconciled_graph, term_scale
from test_gpu_parity import DEV, check_encode, gpu_encode, gpu_graph
from util import Problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vlq():
    import paper_1901_00275_amd as vlq

    vlq.lib()
    return vlq


def _raw_vectors(mix, cfg, ids):
    """Base vectors with the given ids, regenerated chunk by chunk from the seed."""
    ids = np.asarray(ids, np.int64)
    out = np.empty((len(ids), cfg.D), np.float32)
    sizes = {c: cnt for c, cnt in workloads.chunks(cfg)}
    for c in np.unique(ids // datagen.CHUNK):
        X = mix.base_chunk(int(c), DEV, sizes[int(c)])
        sel = np.nonzero(ids // datagen.CHUNK == c)[0]
        rows = torch.as_tensor(ids[sel] % datagen.CHUNK, device=DEV)
        out[sel] = X[rows].cpu().numpy()
        del X
    return out


def _oracle_encode(oracle, pr, X, Sg):
    """Alg. 1 + 2 by the oracle; Sg: the library's graph, whose numbering of tied edges is adopted."""
    cell, _ = oracle.vq_assign(pr.C, X)
    S, E, _ = reconciled_graph(oracle, pr.C, pr.n, cell, Sg)
    return oracle.encode(pr.C, S, E, pr.P, X), S, E


GT_ROWS = 512  # exact ground truth (a brute force over the whole base set) for the first queries only


@pytest.mark.parametrize("name", ["mid_sift", "mid_deep", "billion_sift", "billion_deep"])
def test_full_size_configurations_sampled(vlq, oracle_mod, name):
    cfg = workloads.CONFIGS[name]
    wl = workloads.materialise(vlq, cfg, DEV, log=lambda *a: print(*a, flush=True), gt_rows=GT_ROWS)
    try:
        pr = Problem(cfg.kind, None, wl.Y.cpu().numpy(), wl.C.cpu().numpy(), wl.P.cpu().numpy(), cfg.n)
        rng = np.random.default_rng(7)
        Sg, _ = gpu_graph(vlq, wl.idx, pr)

        # ---- encoding of sampled base vectors ----
        ids = np.sort(rng.choice(cfg.N, 1500, replace=False))
        Xs = _raw_vectors(wl.mix, cfg, ids)
        enc, S, E = _oracle_encode(oracle_mod, pr, Xs, Sg)
        got = gpu_encode(vlq, wl.idx, Xs, cfg.m)
        S, E, _ = reconciled_graph(oracle_mod, pr.C, pr.n, np.concatenate([enc.cell, got[0]]), Sg)
        check_encode(oracle_mod, pr, S, E, Xs, got)
        # the stored lists hold these points with the same fields
        nl = cfg.k * cfg.n
        off = torch.empty(nl + 1, dtype=torch.int64, device=DEV)
        lids = torch.empty(cfg.N, dtype=torch.int32, device=DEV)
        lcodes = torch.empty(cfg.N, cfg.m, dtype=torch.uint8, device=DEV)
        llam = torch.empty(cfg.N, dtype=torch.uint8, device=DEV)
        vlq.vlq_index_get_lists(wl.idx, off, lids, lcodes, llam)
        torch.cuda.synchronize()
        off_h = off.cpu().numpy()
        assert off_h[0] == 0 and off_h[-1] == cfg.N and (np.diff(off_h) >= 0).all()
        for t in rng.choice(len(ids), 200, replace=False):
            label = int(got[0][t]) * cfg.n + int(got[1][t])
            seg = lids[off_h[label]:off_h[label + 1]].cpu().numpy()
            pos = np.searchsorted(seg, ids[t])  # ids ascend inside a list
            assert pos < len(seg) and seg[pos] == ids[t], f"id {ids[t]} not in list {label}"
            assert (np.diff(seg) > 0).all()
            g = off_h[label] + pos
            assert (lcodes[g].cpu().numpy() == got[3][t]).all() and int(llam[g]) == int(got[2][t])
        del lids, lcodes, llam

        # ---- search in the bench launch configuration ----
        nq, w1, w2, K = cfg.nq, cfg.w1[-1], cfg.w2(cfg.w1[-1]), cfg.K
        od = torch.empty(nq, K, device=DEV)
        oi = torch.empty(nq, K, dtype=torch.int32, device=DEV)
        cells = torch.empty(nq, w1, dtype=torch.int32, device=DEV)
        cd = torch.empty(nq, w1, device=DEV)
        sub = torch.empty(nq, w2, dtype=torch.int32, device=DEV)
        ss = torch.empty(nq, w2, device=DEV)
        vlq.vlq_search_debug(wl.idx, wl.Y, nq, w1, w2, K, od, oi, cells, cd, sub, ss)
        torch.cuda.synchronize()
        assert datagen.recall_at(oi[:GT_ROWS], wl.gt[:GT_ROWS], 100) > 0.2  # sanity: the index finds neighbours
        # a query's result does not depend on the batch it arrives in: smaller batches take other kernels (one-pass
        # exact cell selection up to 64 queries, pairwise neighbour products, more column splits and a wider
        # threshold search, scans split over workgroups and merged) and must return the same rows bit for bit
        for nb in (1, 40, 64, 65, 700, 3000):
            bd = torch.full((nb, K), -1.0, device=DEV)
            bi = torch.full((nb, K), -7, dtype=torch.int32, device=DEV)
            vlq.vlq_search(wl.idx, wl.Y[:nb].contiguous(), nb, w1, w2, K, bd, bi)
            torch.cuda.synchronize()
            assert torch.equal(bi, oi[:nb]) and torch.equal(bd, od[:nb]), f"batch of {nb} differs from the full batch"
        qs = np.sort(rng.choice(GT_ROWS, 24, replace=False))
        # the lists these queries visited, as the library stores them, for the oracle's scan
        qs_dev = torch.as_tensor(qs, device=DEV)
        lists = oracle_mod.Lists(*workloads.visited_lists(vlq, wl.idx, cfg, sub[qs_dev]))
        od, oi, cells, cd, sub, ss = (t[torch.as_tensor(qs, device=DEV)].cpu().numpy() for t in (od, oi, cells, cd, sub, ss))
        Yq = pr.Y[qs]
        dist = oracle_mod.coarse(pr.C, Yq)
        ocells = oracle_mod.select_smallest(dist, w1)
        S, E, tied_rows = reconciled_graph(oracle_mod, pr.C, pr.n,
                                           np.concatenate([ocells.ravel(), cells.ravel(), (sub // cfg.n).ravel()]), Sg)
        gt = wl.gt.cpu().numpy()[qs]
        gt_vec = _raw_vectors(wl.mix, cfg, gt)
        gt_enc, Sgt, _ = _oracle_encode(oracle_mod, pr, gt_vec, Sg)
        exact = 0
        for r, q in enumerate(qs):
            what = f"query {q}"
            check_selection(cells[r], dict(enumerate(dist[r])), w1, what=what + " cells")
            assert np.allclose(cd[r], dist[r][cells[r]], rtol=DTOL), what
            score, label = (x[0] for x in oracle_mod.subregion_scores(dist[r:r + 1], S, E, cells[r:r + 1]))
            val = {int(l): float(s) for l, s in zip(label, score)}
            a_max = dist[r][cells[r]].max()
            check_selection(sub[r], val, w2, scale=a_max, what=what + " sub-regions")
            assert np.allclose(ss[r], [val[int(l)] for l in sub[r]], rtol=0, atol=DTOL * a_max), what
            # the whole top-K: the oracle scans the lists the GPU visited, as the library stores them
            o_d, o_i, ncand = (x[0] for x in oracle_mod.scan(pr.C, S, pr.P, lists, Yq[r:r + 1], sub[r:r + 1], K + 16))
            assert ncand == sum(lists.off[l + 1] - lists.off[l] for l in sub[r])
            exact += check_topk(od[r], oi[r], o_d, o_i, K, what=what, scale=term_scale(a_max, Yq[r], pr.C, pr.P), m=cfg.m)
            # every returned point: distance and membership re-derived from its raw vector
            valid = oi[r] >= 0
            assert valid.sum() == K and (np.diff(od[r]) >= 0).all() and len(set(oi[r].tolist())) == K
            Xr = _raw_vectors(wl.mix, cfg, oi[r])
            renc, Sr, _ = _oracle_encode(oracle_mod, pr, Xr, Sg)
            Xh = oracle_mod.reconstruct(pr.C, Sr, pr.P, renc.cell, renc.edge, renc.lamq, renc.codes)
            dref = ((Yq[r].astype(np.float64) - Xh) ** 2).sum(1)
            visited = set(sub[r].tolist())
            for j in range(K):
                tie = renc.cell_d[j, 1] - renc.cell_d[j, 0] <= GAP * renc.cell_d[j, 1] or \
                    renc.edge_d[j, 1] - renc.edge_d[j, 0] <= GAP * renc.cell_d[j, 0]
                if tie:
                    continue  # the point may legitimately sit in a neighbouring list
                assert int(renc.cell[j]) * cfg.n + int(renc.edge[j]) in visited, f"{what}: result {j} from an unvisited list"
                frac = renc.lam_coord[j] - np.floor(renc.lam_coord[j])
                if abs(frac - 0.5) < LAM_WINDOW or (renc.code_d[j, :, 1] - renc.code_d[j, :, 0] <= GAP * renc.code_d[j, :, 1]).any():
                    continue  # byte / code inside a tie band: the stored code may differ
                assert abs(od[r][j] - dref[j]) <= DTOL * dref[j], f"{what}: distance of result {j}"
            # completeness: the true neighbour, if visited and good enough, must be returned
            glabel = int(gt_enc.cell[r]) * cfg.n + int(gt_enc.edge[r])
            gh = oracle_mod.reconstruct(pr.C, Sgt, pr.P, gt_enc.cell[r:r + 1], gt_enc.edge[r:r + 1],
                                        gt_enc.lamq[r:r + 1], gt_enc.codes[r:r + 1])
            gd = ((Yq[r].astype(np.float64) - gh[0]) ** 2).sum()
            if glabel in visited and gd < od[r][K - 1] * (1 - 1e-4):
                assert gt[r] in set(oi[r].tolist()), f"{what}: true neighbour {gt[r]} missed"
        print(f"[{name}] {len(qs)} sampled queries: full top-{K} inside the parity bands, {exact} with id sets identical "
              f"to the oracle's scan of the same lists; {tied_rows} graph rows of their cells numbered by a tie", flush=True)
    finally:
        vlq.vlq_index_free(wl.idx)
