#!/usr/bin/env python3
"""Benchmark of the VLQ-ADC query path on one MI355X.

A step is one vlq_search call (all of Alg. 3: coarse distances, cell and
sub-region selection, lookup tables, list scan, K-selection) over the whole
query batch of the configuration, with queries and index resident in HBM.
Prints one JSON line: queries/s at the stated recall, the roofline figures of
the dominant kernel (the list scan) from HIP events on the search stream, and
the CPU oracle's timing on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def scan_bytes(vlq, wl, w1, w2, torch):
    """Algorithmic bytes of the list scan for one batch: every point of every visited list once
    (m code bytes + 1 lambda byte + 4 bytes of the stored query-independent term) plus the two
    list offsets (8 bytes) of every visited list.  Also returns the traversal and the results of
    that search (device tensors) for the parity sample."""
    cfg = wl.cfg
    nq = wl.Y.shape[0]
    dev = wl.Y.device
    od = torch.empty(nq, cfg.K, device=dev)
    oi = torch.empty(nq, cfg.K, dtype=torch.int32, device=dev)
    cells = torch.empty(nq, w1, dtype=torch.int32, device=dev)
    cd = torch.empty(nq, w1, device=dev)
    sub = torch.empty(nq, w2, dtype=torch.int32, device=dev)
    ss = torch.empty(nq, w2, device=dev)
    vlq.vlq_search_debug(wl.idx, wl.Y, nq, w1, w2, cfg.K, od, oi, cells, cd, sub, ss)
    off = torch.empty(cfg.k * cfg.n + 1, dtype=torch.int64, device=dev)
    vlq.vlq_index_get_lists(wl.idx, off, None, None, None)
    torch.cuda.synchronize()
    s = sub.long().clamp_min(0)
    lens = (off[s + 1] - off[s]) * (sub >= 0)
    points = int(lens.sum())
    visited = int((sub >= 0).sum())
    return points * (cfg.m + 5) + visited * 8, points, (od, oi, cells, cd, sub, ss)


def parity_on_sample(vlq, wl, w1, w2, dbg, torch, nsample=100, qlam=None):
    """The tests' protocol on the first queries of the timed batch, at full size: cells, sub-regions
    and scores against the oracle's traversal, and the whole top-K against the oracle's scan of the
    lists the GPU visited (copied out of the library).  Returns the summary and the list of
    violations (empty when the sample is inside the parity bands)."""
    import numpy as np

    import oracle
    from datagen import workloads

    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from parity import DTOL, check_selection, check_topk, reconciled_graph, term_scale

    cfg = wl.cfg
    prm = vlq.vlq_index_params(wl.idx)
    grid = (float(prm.lambda_lo), float(prm.lambda_hi))  # the lambda byte grid of this index
    ns = min(nsample, wl.Y.shape[0])
    od, oi, cells, cd, sub, ss = (t[:ns] for t in dbg)
    lists = oracle.Lists(*workloads.visited_lists(vlq, wl.idx, cfg, sub))
    od, oi, cells, cd, sub, ss = (t.cpu().numpy() for t in (od, oi, cells, cd, sub, ss))
    Cb, P, Y = wl.C.cpu().numpy(), wl.P.cpu().numpy(), wl.Y[:ns].cpu().numpy()
    dist = oracle.coarse(Cb, Y)
    ocells = oracle.select_smallest(dist, w1)
    Sd = torch.empty(cfg.k, cfg.n, dtype=torch.int32, device=wl.Y.device)
    vlq.vlq_index_get_graph(wl.idx, Sd, None)
    torch.cuda.synchronize()
    S, E, _ = reconciled_graph(oracle, Cb, cfg.n, np.concatenate([ocells.ravel(), cells.ravel(), (sub[sub >= 0] // cfg.n).ravel()]),
                               Sd.cpu().numpy())
    ids_exact = tie = 0
    max_rel = 0.0
    bad = []
    for q in range(ns):
        try:
            same_c = check_selection(cells[q], dict(enumerate(dist[q])), w1, what=f"query {q} cells")
            assert np.allclose(cd[q], dist[q][cells[q]], rtol=DTOL), f"query {q} cell distances"
            score, label = (x[0] for x in oracle.subregion_scores(dist[q:q + 1], S, E, cells[q:q + 1], qlam or (-np.inf, np.inf)))
            val = {int(l): float(v) for l, v in zip(label, score)}
            a_max = dist[q][cells[q]].max()
            same_s = check_selection(sub[q], val, w2, scale=a_max, what=f"query {q} sub-regions")
            assert np.allclose(ss[q], [val[int(l)] for l in sub[q]], rtol=0, atol=DTOL * a_max), f"query {q} scores"
            o_d, o_i, _ = (x[0] for x in oracle.scan(Cb, S, P, lists, Y[q:q + 1], sub[q:q + 1], cfg.K + 16, *grid))
            same_k = check_topk(od[q], oi[q], o_d, o_i, cfg.K, what=f"query {q}", scale=term_scale(a_max, Y[q], Cb, P), m=cfg.m)
            o_map = {int(i): float(d) for d, i in zip(o_d, o_i)}
            max_rel = max(max_rel, max(abs(float(g) - o_map[int(i)]) / max(o_map[int(i)], 1e-30) for g, i in zip(od[q], oi[q]) if i >= 0))
            if same_c and same_s and same_k and (oi[q] == o_i[:cfg.K]).all():
                ids_exact += 1
            else:
                tie += 1
        except AssertionError as e:
            bad.append(str(e)[:200])
    return {"queries": ns, "ids_exact": ids_exact, "in_tie_band": tie, "violations": len(bad),
            "max_rel_dist_err": max_rel}, bad


def cpu_baseline(vlq, wl, w1, w2, torch, target_s=15.0):
    """The oracle's search (as it stands) on the host cores, on a sample of the
    batch's queries, against the same index (copied out of the library for this
    timing leg only; nothing is compared against it for parity)."""
    import numpy as np

    import oracle

    cfg = wl.cfg
    dev = wl.Y.device
    N = vlq.vlq_index_ntotal(wl.idx)
    off = torch.empty(cfg.k * cfg.n + 1, dtype=torch.int64, device=dev)
    ids = torch.empty(N, dtype=torch.int32, device=dev)
    codes = torch.empty(N, cfg.m, dtype=torch.uint8, device=dev)
    lam = torch.empty(N, dtype=torch.uint8, device=dev)
    vlq.vlq_index_get_lists(wl.idx, off, ids, codes, lam)
    torch.cuda.synchronize()
    lists = oracle.Lists(off.cpu().numpy(), ids.cpu().numpy(), codes.cpu().numpy(), lam.cpu().numpy())
    del ids, codes, lam
    Cb, P, Y = wl.C.cpu().numpy(), wl.P.cpu().numpy(), wl.Y.cpu().numpy()

    # graph rows are index data, not query work: for this timing leg they are copied out of the
    # library as well (the oracle's own graph construction is O(k^2 D) and would take minutes here)
    Sd = torch.empty(cfg.k, cfg.n, dtype=torch.int32, device=dev)
    Ed = torch.empty(cfg.k, cfg.n, dtype=torch.float32, device=dev)
    vlq.vlq_index_get_graph(wl.idx, Sd, Ed)
    torch.cuda.synchronize()
    S, E = Sd.cpu().numpy(), Ed.cpu().numpy().astype(np.float64)

    def run(Yq):
        t0 = time.time()
        dist = oracle.coarse(Cb, Yq)
        cells = oracle.select_smallest(dist, w1)
        score, label = oracle.subregion_scores(dist, S, E, cells)
        sub = oracle.select_smallest(score, w2, key=label)
        out_d, out_i, _ = oracle.scan(Cb, S, P, lists, Yq, sub, cfg.K)
        return time.time() - t0, out_i

    nprobe = min(32, len(Y))
    t, _ = run(Y[:nprobe])
    ns = int(min(len(Y), max(nprobe, target_s / max(t / nprobe, 1e-9))))
    t, out_i = run(Y[:ns])
    cores = oracle.num_threads()
    cpu = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    base = {"value": ns / t, "unit": "queries/s", "cores": cores, "kind": "oracle", "cpu": cpu,
            "sample": f"first {ns} of the {len(Y)} queries, index and graph copied from the library, same w1/w2/K; {t:.1f} s of oracle search"}
    if cores > 1:  # the same code on one thread, on a sample sized for about a third of the time
        n1 = int(min(ns, max(4, ns / cores * 0.35)))
        oracle.set_num_threads(1)
        try:
            t1, _ = run(Y[:n1])
        finally:
            oracle.set_num_threads(cores)
        base["one_core"] = {"value": n1 / t1, "unit": "queries/s", "cores": 1,
                            "sample": f"first {n1} queries, {t1:.1f} s"}
    return base, out_i, ns


def measured_traffic(workload):
    """HBM bytes per launch of the scan kernel from the committed counter summary of this workload
    (two rocprofv3 --pmc runs of this script, scaled by the copy yardstick), and the name of that
    file; (None, None) if there is none.  Not measured in this run: counters need the profiler."""
    name = f"profiles/k_scan_stream_{workload}_hbm_traffic.md"
    try:
        for line in open(os.path.join(ROOT, name)):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1])), name
    except OSError:
        pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="billion_sift")
    ap.add_argument("--w1", type=int, default=0, help="probed cells (default: the configuration's operating point)")
    ap.add_argument("--points", type=int, default=0, help="build only the first POINTS vectors (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="also the alpha, batch-size and K sweeps of the configuration (the w1 sweep always runs)")
    ap.add_argument("--query-lambda", default="",
                    help="restrict the query's lambda in the region traversal to LO,HI (Sec. 3.3.1 variant; 'grid' = the "
                         "range of the lambda byte, '0,1' = the segment between the two centroids; default: the whole line)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain streaming kernel of known size (torch.frac over 2^28 floats: 1 GiB read, "
                         "1 GiB written), the yardstick for the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1")
        sys.exit(2)

    import torch

    import datagen
    import paper_1901_00275_amd as vlq
    from datagen import workloads

    vlq.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[args.config]
    wl = workloads.materialise(vlq, cfg, "cuda:0", n_points=args.points or None, log=log)
    nq, K = cfg.nq, cfg.K
    dev = wl.Y.device
    qlam = None
    if args.query_lambda:
        prm = vlq.vlq_index_params(wl.idx)
        qlam = (prm.lambda_lo, prm.lambda_hi) if args.query_lambda == "grid" else tuple(float(x) for x in args.query_lambda.split(","))
        vlq.vlq_index_set_query_lambda_range(wl.idx, *qlam)
    od = torch.empty(nq, K, device=dev)
    oi = torch.empty(nq, K, dtype=torch.int32, device=dev)

    def timed(w1, steps, warmup, w2=None):
        w2 = w2 or cfg.w2(w1)
        for _ in range(warmup):
            vlq.vlq_search(wl.idx, wl.Y, nq, w1, w2, K, od, oi)
        torch.cuda.synchronize()
        vlq.vlq_profile_read(wl.idx)
        vlq.vlq_profile_enable(wl.idx, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            vlq.vlq_search(wl.idx, wl.Y, nq, w1, w2, K, od, oi)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        vlq.vlq_profile_enable(wl.idx, False)
        prof = vlq.vlq_profile_read(wl.idx)
        rec = {f"R@{r}": datagen.recall_at(oi, wl.gt, r) for r in (1, 10, 100)}
        return dt, prof, rec, w2

    w1 = args.w1 or cfg.w1[-1]
    dt, prof, rec, w2 = timed(w1, args.steps, args.warmup)
    nbytes, points, dbg = scan_bytes(vlq, wl, w1, w2, torch)
    scan_ms, scan_launches = prof["scan"]
    scan_avg_s = scan_ms / 1e3 / max(scan_launches, 1)
    achieved = nbytes / scan_avg_s / 1e9
    stage_ms = {s: round(v[0] / args.steps, 4) for s, v in prof.items()}
    traffic, traffic_source = measured_traffic(cfg.name)
    # coarse distances (Alg. 3, first loop): 2 nq k D flop of the contraction per step, against the bf16 matrix peak
    coarse_flop = 2.0 * nq * cfg.k * cfg.D
    coarse_s = prof["coarse"][0] / 1e3 / args.steps
    result = {
        "metric": "queries/sec at Recall@10 (1B pts, 1 GPU); ADC-scan HBM GB/s vs peak",
        "value": nq * args.steps / dt,
        "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "N": vlq.vlq_index_ntotal(wl.idx), "D": cfg.D, "centroids": cfg.k,
                   "edges": cfg.n, "code_bytes": cfg.m, "queries": nq, "w1": w1, "w2": w2, "K": K,
                   "query_lambda_range": qlam,
                   "recall": rec, "points_scanned_per_query": points / nq,
                   "stage_ms_per_step": stage_ms, "build_s": wl.timings,
                   "coarse_mfma": {"flop_per_step": coarse_flop, "ms_per_step": coarse_s * 1e3,
                                   "achieved_tflops": coarse_flop / max(coarse_s, 1e-12) / 1e12,
                                   "peak_tflops": BF16_PEAK_TFLOPS,
                                   "frac": coarse_flop / max(coarse_s, 1e-12) / 1e12 / BF16_PEAK_TFLOPS,
                                   "note": "2 nq k D flop of Alg. 3's first loop over the time of both sweeps of the "
                                           "bf16 product (hi parts of the split operands; the first sweep visits every other tile)"}},
        "roofline": {"bound": "hbm", "kernel": "k_scan_stream", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": scan_avg_s * 1e3,
                     "bytes_note": "(m + 5) bytes per scanned point + 8 bytes of list offsets per visited list; the kernel "
                                   "itself reads a 16-byte descriptor per list (offset, length and the two coarse "
                                   "distances of Eq. 17), not counted beyond the 8"},
    }
    if args.copy_calibration:
        src = torch.rand(1 << 28, device=dev)
        dst = torch.empty_like(src)
        torch.frac(src, out=dst)
        torch.cuda.synchronize()
        del src, dst
    # the (w1, queries/s, Recall@10) curve of the configuration; the headline is its last point
    sweep = []
    for w in cfg.w1:
        reps = max(3, args.steps // 2)
        d2, p2, r2, w22 = timed(w, reps, 1)
        pts = scan_bytes(vlq, wl, w, w22, torch)[1]
        sweep.append({"w1": w, "w2": w22, "queries_per_s": nq * reps / d2, "ms_per_step": d2 / reps * 1e3,
                      "points_scanned_per_query": pts / nq, **r2})
    result["config"]["sweep"] = sweep
    # the cheapest probe whose Recall@10 is within 5 % of the headline operating point's
    ref = rec["R@10"]
    ok = [e for e in sweep if e["R@10"] >= 0.95 * ref]
    if ok:
        best = max(ok, key=lambda e: e["queries_per_s"])
        result["config"]["cheapest_within_5pct_of_R@10"] = {"w1": best["w1"], "w2": best["w2"],
                                                             "queries_per_s": best["queries_per_s"], "R@10": best["R@10"]}
    if args.sweep:
        # the share alpha of the w1 * n sub-regions that is scanned (Sec. 5, parameter study), at the headline w1
        if not cfg.w2_fixed and cfg.n > 1:
            asw = []
            for alpha in (0.25, 0.4, 0.5):
                w2a = max(1, int(alpha * w1 * cfg.n))
                d2, p2, r2, _ = timed(w1, max(2, args.steps // 2), 1, w2a)
                asw.append({"alpha": alpha, "w1": w1, "w2": w2a, "queries_per_s": nq * max(2, args.steps // 2) / d2, **r2})
            result["config"]["alpha_sweep"] = asw
        # batch-size and K sweeps of the configuration (at the headline w1): the first nb queries of the batch
        bs = []
        for nb in cfg.batches:
            for Kx in (cfg.Ks or (K,)):
                Yb = wl.Y[:nb].contiguous()
                odb = torch.empty(nb, Kx, device=dev)
                oib = torch.empty(nb, Kx, dtype=torch.int32, device=dev)
                reps = 20 if nb <= 256 else max(2, args.steps // 2)
                for _ in range(2):
                    vlq.vlq_search(wl.idx, Yb, nb, w1, w2, Kx, odb, oib)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(reps):
                    vlq.vlq_search(wl.idx, Yb, nb, w1, w2, Kx, odb, oib)
                torch.cuda.synchronize()
                d3 = (time.perf_counter() - t0) / reps
                bs.append({"queries": nb, "K": Kx, "ms_per_call": d3 * 1e3, "queries_per_s": nb / d3,
                           f"R@{Kx}": datagen.recall_at(oib, wl.gt[:nb], Kx)})
        if bs:
            result["config"]["batch_sweep"] = bs
    violations = []
    if not args.no_cpu_baseline:
        summary, violations = parity_on_sample(vlq, wl, w1, w2, dbg, torch, qlam=qlam)
        result["config"]["parity_on_sample"] = summary
        base, o_ids, ns = cpu_baseline(vlq, wl, w1, w2, torch)
        result["cpu_baseline"] = base
    print(json.dumps(result), flush=True)
    vlq.vlq_index_free(wl.idx)
    if violations:
        for v in violations[:10]:
            log("bench.py: parity violation on the sample:", v)
        sys.exit(1)


if __name__ == "__main__":
    main()
