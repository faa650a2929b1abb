"""Throughput of the PQTopK hot path on one MI355X.

A step is one pass of the whole path over one batch: pq_subitem_scores (Eq. 4) then pq_score_topk (Eq. 5 +
TopK, Algorithm 1) for B queries against the whole catalogue, inputs resident in HBM.  The default workload is
the Gowalla-shaped catalogue (N = 1.28M items, d = 512, m = 8, b = 256, K = 10) at batch 1, on seeded
synthetic data.  One JSON line is printed.
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

HBM_PEAK_GBS = 8000.0        # MI355X published HBM3E bandwidth
LDS_PEAK_GBS = 128 * 256 * 2.4   # 128 B/clk/CU x 256 CUs x 2.4 GHz: what the LDS can return per second


def cpu_baseline(G, cent, Q, K, budget_s=12.0):
    """The CPU oracle as it stands, timed on this host on whole-catalogue queries (bounded sample): on all host
    threads (the reported baseline) and, for a few seconds, on one."""
    import numpy as np
    from oracle import pq_oracle
    threads = pq_oracle.num_threads()
    q1 = np.ascontiguousarray(Q[:1])
    N = G.shape[0]

    def run(budget):
        pq_oracle.pqtopk(G, cent, q1, K)                  # warm-up
        t0 = time.perf_counter()
        n = 0
        while True:
            pq_oracle.pqtopk(G, cent, q1, K)
            n += 1
            el = time.perf_counter() - t0
            if el > budget or n >= 200:
                return n, el

    n, el = run(budget_s)
    pq_oracle.set_num_threads(1)
    try:
        n1, el1 = run(3.0)
    finally:
        pq_oracle.set_num_threads(threads)
    return {"value": N * n / el, "unit": "items/s", "queries_per_s": n / el, "cores": threads, "kind": "oracle",
            "sample": f"{n} single-query passes of the oracle (Eq. 4, Eq. 5 over all {N} items, TopK) in {el:.2f} s",
            "one_thread_items_per_s": N * n1 / el1}


def measured_traffic(workload: str):
    """HBM bytes per scan launch of this workload as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, each scaled by a
    plain copy of known size), with where the figure comes from.  Counters cannot be read in-process: the figure is the
    one recorded in profiles/pmc_traffic.json from the --pmc runs whose summaries lie beside it (it describes the
    kernel as it was when those runs were made), or None for a workload that has not been profiled."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f).get(workload)
    except (OSError, ValueError):
        rec = None
    if not rec:
        return None, "not profiled: no rocprofv3 --pmc run of this workload is recorded in profiles/pmc_traffic.json"
    return rec.get("traffic_bytes_per_launch"), \
        f"recorded, not measured by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in {rec.get('source')}"


def measured_lds_peak(pq, torch):
    """Random 16-byte gathers from a 32 KB table in LDS, 16 waves per CU (the batched scan's lookup pattern with nothing
    else going on), measured now: GB/s over the whole chip."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    rounds = 16 * 256
    best = 0.0
    for threads, per_cu in ((512, 2), (1024, 1)):
        pq.pq_measure_lds_gather(16, 32768, rounds, False, cus * per_cu, threads, 3, sink)
        ms = sorted(pq.pq_measure_lds_gather(16, 32768, rounds, False, cus * per_cu, threads, 10, sink) for _ in range(5))[2]
        best = max(best, cus * per_cu * threads * rounds * 16.0 / (ms * 1e-3) / 1e9)
    return best


def sweep(args):
    """Catalogue-size sweep in the manner of Section 5 (RQ2, Figure 2): random model output, random sub-item
    embeddings and codes, m = 8 and m = 64, batch 1, K = 10, N from 10^3 up to what --sweep-max-bytes of codes
    allows.  Per point: whole-step time (Eq. 4 + Eq. 5 + TopK), the scan kernel's duration and its share of the HBM
    roofline; results are checked against the oracle where the code matrix is at most --sweep-check-bytes."""
    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W
    from oracle import pq_oracle

    d, b, K, B = 512, 256, 10, 1
    points = []
    for m in (8, 64):
        cent = W.centroids(m, b, d, seed=m)
        Q = W.queries(B, d, seed=m)
        Cd, Qd = torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
        for e in range(3, 10):
            N = 10 ** e
            if N * m > args.sweep_max_bytes:
                continue
            Gd = W.codes_uniform_device(N, m, b, seed=e)
            sub = pq.PreparedSubitemScores(Qd, Cd)
            checked = N * m <= args.sweep_check_bytes
            if not checked:
                # too large for the oracle: the very last item gets the best sub-id of every split, so it must come
                # back first, with the score the oracle gives that one row (all byte offsets of the scan are exercised)
                sub()
                torch.cuda.synchronize()
                S_host = sub.S.cpu().numpy()
                best_row = S_host[0].argmax(axis=1).astype(np.uint8)
                Gd[N - 1] = torch.from_numpy(best_row).cuda()
            top = pq.PreparedScoreTopK(Gd, sub.S, K)
            for _ in range(3):
                sub(); top()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sub(); top()
            torch.cuda.synchronize()
            once = time.perf_counter() - t0
            steps = int(max(5, min(2000, 0.25 / max(once, 1e-6))))
            t0 = time.perf_counter()
            for _ in range(steps):
                sub(); top()
            torch.cuda.synchronize()
            el = (time.perf_counter() - t0) / steps
            n_prof = max(3, min(50, steps))
            t_warm = time.perf_counter()                     # (untimed: the scan kernel alone until the clocks have settled)
            while time.perf_counter() - t_warm < 0.02:
                pq.pq_score_topk_profile(Gd, sub.S, K, n_prof, workspace=top.workspace)
            scan_ms = sorted(pq.pq_score_topk_profile(Gd, sub.S, K, n_prof, workspace=top.workspace) for _ in range(5))[2]
            parity, planted = None, None
            if checked:
                rid, rsc = pq_oracle.score_topk(Gd.cpu().numpy(), sub.S.cpu().numpy(), K)
                parity = bool(np.array_equal(top.ids.cpu().numpy(), rid) and
                              np.array_equal(top.scores.cpu().numpy().view(np.uint32), rsc.view(np.uint32)))
            else:
                want = pq_oracle.item_scores(best_row[None, :], S_host[0])
                planted = bool(int(top.ids[0, 0]) == N - 1 and
                               np.array_equal(top.scores.cpu().numpy()[0, :1].view(np.uint32), want.view(np.uint32)))
            gbs = N * m / (scan_ms * 1e-3) / 1e9
            pt = {"N": N, "m": m, "us_per_step": el * 1e6, "items_per_s": N / el, "scan_kernel_us": scan_ms * 1e3,
                  "scan_GBps": gbs, "hbm_frac": gbs / HBM_PEAK_GBS, "parity_vs_oracle": parity,
                  "planted_winner_found": planted}
            points.append(pt)
            print(f"m={m:2d} N={N:>10d}  step {el * 1e6:10.1f} us  {N / el / 1e9:7.3f} Gitem/s  scan {scan_ms * 1e3:10.1f} us "
                  f"{gbs:7.0f} GB/s ({100 * gbs / HBM_PEAK_GBS:4.1f} % of HBM peak)  "
                  + (f"parity {parity}" if checked else f"planted winner found {planted}"), file=sys.stderr, flush=True)
            del sub, top, Gd
            torch.cuda.empty_cache()
    best = max(points, key=lambda p: p["items_per_s"])
    print(json.dumps({
        "metric": "items scored/sec (PQTopK, whole path incl. top-K), catalogue-size sweep", "value": best["items_per_s"],
        "unit": "items/s", "n_gpus": 1, "higher_is_better": True, "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": {"workload": f"sweep: d={d} b={b} K={K} batch={B}, m in (8, 64), N = 10^3..10^9, "
                                                    "uniform codes drawn on the device"},
        "sweep": points}))


def compare(args):
    """The paper's three-way comparison (Table 3, scoring time per user, TopK included) on the Gowalla-shaped workload:
    PQTopK (Algorithm 1) against RecJPQ's split-major scoring (Algorithm 2) and the default matrix-vector scoring
    over reconstructed item embeddings (Eq. 2 + Eq. 3), all on this GPU, batch 1."""
    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W
    from oracle import pq_oracle

    cfg = W.CONFIGS[args.config]
    G, cent, Q = W.make(cfg, B=1)
    N, m, b, K, d = cfg.N, cfg.m, cfg.b, cfg.K, cfg.d
    Gd, Cd, Qd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
    sub = pq.PreparedSubitemScores(Qd, Cd)
    top = pq.PreparedScoreTopK(Gd, sub.S, K)
    Wd = pq.pq_reconstruct_items(Gd, Cd)                          # built once, as an index would be
    scores = torch.empty((1, (N + 3) // 4 * 4), dtype=torch.float32, device="cuda")
    ws = torch.empty(pq.pq_topk_scores_workspace_bytes(N, 1, K), dtype=torch.uint8, device="cuda")
    ids2 = torch.empty((1, K), dtype=torch.int32, device="cuda"); sc2 = torch.empty((1, K), dtype=torch.float32, device="cuda")
    ids3 = torch.empty_like(ids2); sc3 = torch.empty_like(sc2)

    def pqtopk():
        sub(); top()

    def recjpq():
        sub()
        pq.pq_recjpq_scores(Gd, sub.S, out=scores)
        pq.pq_topk_scores(scores, K, N=N, workspace=ws, out_ids=ids2, out_scores=sc2)

    def default():
        pq.pq_default_scores(Wd, Qd, out=scores)
        pq.pq_topk_scores(scores, K, N=N, workspace=ws, out_ids=ids3, out_scores=sc3)

    def timed(fn, steps):
        for _ in range(max(50, steps // 4)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    t_pq = timed(pqtopk, 2000)
    t_rj = timed(recjpq, 1000)
    t_df = timed(default, 200)
    rid, rsc = pq_oracle.pqtopk(G, cent, Q, K)
    same = lambda a: bool(np.array_equal(a.cpu().numpy(), rid))
    out = {
        "metric": "scoring time per query incl. top-K: PQTopK vs RecJPQScore (Algorithm 2) vs Default (W phi)",
        "value": N / t_pq, "unit": "items/s", "n_gpus": 1, "higher_is_better": True, "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N} d={d} m={m} b={b} K={K} batch=1, codes {cfg.codes}, seed {cfg.seed}"},
        "comparison": {
            "pqtopk": {"us_per_query": t_pq * 1e6, "ids_equal_oracle": same(top.ids)},
            "recjpq_algorithm2": {"us_per_query": t_rj * 1e6, "ids_equal_oracle": same(ids2),
                                  "scores_bit_equal_pqtopk": bool(torch.equal(sc2, top.scores))},
            "default_matvec": {"us_per_query": t_df * 1e6, "topk_overlap_with_oracle": int(len(set(ids3.cpu().numpy()[0]) & set(rid[0]))),
                               "embedding_matrix_bytes": int(N) * d * 4},
            "speedup_over_recjpq": t_rj / t_pq, "speedup_over_default": t_df / t_pq,
        },
    }
    print(json.dumps(out))


def subset_mode(args):
    """Algorithm 1 with a candidate list V: GPU time per call (HIP events around back-to-back calls) over list sizes on
    --config's catalogue at batch 1, for lists in random order and in ascending order, with the result checked
    against the oracle."""
    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W
    from oracle import pq_oracle

    cfg = W.CONFIGS[args.config]
    G, cent, Q = W.make(cfg, B=1)
    N, m, b, K = cfg.N, cfg.m, cfg.b, cfg.K
    Gd = torch.from_numpy(G).cuda()
    S = pq.pq_subitem_scores(torch.from_numpy(Q).cuda(), torch.from_numpy(cent).cuda())
    Sh = S.cpu().numpy()
    points = []
    for n in [x for x in (10 ** 3, 10 ** 4, 10 ** 5, 10 ** 6, N) if x <= N]:
        for ascending in (False, True):
            V = W.candidate_list(N, n, seed=n, ascending=ascending)
            Vd = torch.from_numpy(V).cuda()
            call = pq.PreparedScoreTopKSubset(Gd, S, Vd, K)
            ids, sc = call.ids, call.scores
            for _ in range(300):
                call()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(300):
                call()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / 300 * 1e3
            rid, rsc = pq_oracle.score_topk_subset(G, Sh, V, K)
            ok = bool(np.array_equal(ids.cpu().numpy(), rid) and
                      np.array_equal(sc.cpu().numpy().view(np.uint32), rsc.view(np.uint32)))
            pt = {"list_size": n, "order": "ascending" if ascending else "random", "us_per_call": us,
                  "items_per_s": n / (us * 1e-6), "gathered_GBps": n * m / (us * 1e-6) / 1e9, "parity_vs_oracle": ok}
            points.append(pt)
            print(f"|V|={n:>8d} {pt['order']:9s} {us:8.2f} us  {pt['items_per_s'] / 1e9:7.2f} Gitem/s  parity {ok}",
                  file=sys.stderr, flush=True)
    best = max(points, key=lambda p: p["items_per_s"])
    print(json.dumps({
        "metric": "items scored/sec with a candidate list (Algorithm 1's V), top-K included", "value": best["items_per_s"],
        "unit": "items/s", "n_gpus": 1, "higher_is_better": True, "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N} m={m} b={b} K={K} batch=1, seeded candidate lists of 10^3 .. N items"},
        "subset": points}))


def wide_mode(args):
    """Codebooks with 16-bit sub-ids (pq_score_topk_u16): alphabets of 1024 to 8192 sub-ids per split, batch 1, K = 10,
    catalogues from the headline size up to 5*10^7 items.  Per point: whole-step time (Eq. 4 + Eq. 5 + TopK), the scan
    kernel's duration and its share of the HBM roofline over the 2*N*m bytes of codes; results are checked against the
    oracle where the code matrix is at most --sweep-check-bytes."""
    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W
    from oracle import pq_oracle

    d, K, B = 512, 10, 1
    points = []
    for (m, b) in ((8, 1024), (8, 4096), (4, 8192), (16, 2048), (12, 1024)):
        cent = W.centroids(m, b, d if d % m == 0 else 32 * m, seed=m + b)
        Q = W.queries(B, cent.shape[0] * cent.shape[2], seed=m + b)
        Cd, Qd = torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
        for N in (1_280_000, 10_000_000, 50_000_000):
            if 2 * N * m > args.sweep_max_bytes:
                continue
            Gd = W.codes_uniform_u16_device(N, m, b, seed=N % 1000 + m)
            sub = pq.PreparedSubitemScores(Qd, Cd)
            top = pq.PreparedScoreTopKU16(Gd, sub.S, K)
            for _ in range(3):
                sub(); top()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            sub(); top()
            torch.cuda.synchronize()
            once = time.perf_counter() - t0
            steps = int(max(5, min(2000, 0.25 / max(once, 1e-6))))
            t0 = time.perf_counter()
            for _ in range(steps):
                sub(); top()
            torch.cuda.synchronize()
            el = (time.perf_counter() - t0) / steps
            scan_ms = pq.pq_score_topk_u16_profile(Gd, sub.S, K, max(3, min(50, steps)), workspace=top.workspace)
            parity = None
            if 2 * N * m <= args.sweep_check_bytes:
                rid, rsc = pq_oracle.score_topk_u16(Gd.cpu().numpy(), sub.S.cpu().numpy(), K)
                parity = bool(np.array_equal(top.ids.cpu().numpy(), rid) and
                              np.array_equal(top.scores.cpu().numpy().view(np.uint32), rsc.view(np.uint32)))
            gbs = 2 * N * m / (scan_ms * 1e-3) / 1e9
            pt = {"N": N, "m": m, "b": b, "us_per_step": el * 1e6, "items_per_s": N / el, "scan_kernel_us": scan_ms * 1e3,
                  "scan_GBps": gbs, "hbm_frac": gbs / HBM_PEAK_GBS, "parity_vs_oracle": parity}
            points.append(pt)
            print(f"m={m:2d} b={b:5d} N={N:>10d}  step {el * 1e6:9.1f} us  {N / el / 1e9:7.3f} Gitem/s  scan {scan_ms * 1e3:9.1f} us "
                  f"{gbs:7.0f} GB/s ({100 * gbs / HBM_PEAK_GBS:4.1f} % of HBM peak)  parity {parity}", file=sys.stderr,
                  flush=True)
            del sub, top, Gd
            torch.cuda.empty_cache()
    best = max(points, key=lambda p: p["items_per_s"])
    print(json.dumps({
        "metric": "items scored/sec (PQTopK over 16-bit sub-ids, whole path incl. top-K)", "value": best["items_per_s"],
        "unit": "items/s", "n_gpus": 1, "higher_is_better": True, "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "config": {"workload": f"16-bit sub-ids: K={K} batch={B}, (m, b) in (8, 1024), (8, 4096), (4, 8192), "
                                                    "(16, 2048), (12, 1024), N = 1.28M, 10^7, 5*10^7, uniform codes drawn on "
                                                    "the device"},
        "wide": points}))


def variants_mode(args):
    """The step of --config at batch 1 under each choice of kernels the library has for a small K: the short scan and
    the small fold (what it runs), and each of them replaced by the general kernel (pq_measure_force_general).  Every
    variant: steady-state time per step over --steps steps, parity with the oracle, one step at a time.  Run under
    rocprofv3 --kernel-trace --stats, the kernels of all variants show up under their own names."""
    import numpy as np
    import torch
    from oracle import pq_oracle
    from paper_2408_09992_amd import binding as pq, workloads as W

    cfg = W.CONFIGS[args.config]
    G, cent, Q = W.make(cfg, B=1)
    N, m, b, d = cfg.N, cfg.m, cfg.b, cfg.d
    Gd, Cd, Qd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
    Sd = torch.empty((1, m, b), dtype=torch.float32, device="cuda")
    rows = []
    names = {0: "short scan + small fold (the library's choice)", 1: "general scan + small fold", 2: "short scan + general fold",
             3: "general scan + general fold"}
    try:
        for K in (1, 10, 31):
            rid, rsc = pq_oracle.pqtopk(G, cent, Q, K)
            for mask in (0, 1, 2, 3):
                pq.pq_measure_force_general(mask)
                ws = torch.empty(pq.pq_score_topk_workspace_bytes(N, 1, m, b, K), dtype=torch.uint8, device="cuda")
                ids = torch.empty((1, K), dtype=torch.int32, device="cuda")
                sc = torch.empty((1, K), dtype=torch.float32, device="cuda")
                sub = pq.PreparedSubitemScores(Qd, Cd, out=Sd)
                top = pq.PreparedScoreTopK(Gd, Sd, K, workspace=ws, out_ids=ids, out_scores=sc)
                t_warm = time.perf_counter()
                while time.perf_counter() - t_warm < 0.05:
                    for _ in range(200):
                        sub(); top()
                    torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    sub(); top()
                torch.cuda.synchronize()
                us = (time.perf_counter() - t0) / args.steps * 1e6
                lat = []
                for _ in range(200):
                    t1 = time.perf_counter()
                    sub(); top()
                    torch.cuda.synchronize()
                    lat.append((time.perf_counter() - t1) * 1e6)
                parity = bool(np.array_equal(ids.cpu().numpy(), rid) and
                              np.all(np.abs(sc.cpu().numpy() - rsc) <= 1e-5 * np.maximum(np.abs(rsc), 1.0)))
                rows.append({"K": K, "variant": names[mask], "mask": mask, "us_per_step": us,
                             "one_at_a_time_median_us": float(np.median(lat)), "parity_vs_oracle": parity})
                print(f"K={K:3d} {names[mask]:48s} {us:7.2f} us/step  one at a time {np.median(lat):7.2f} us  parity {parity}",
                      file=sys.stderr, flush=True)
    finally:
        pq.pq_measure_force_general(0)
    best = min(r["us_per_step"] for r in rows if r["K"] == 10)
    print(json.dumps({"metric": "step time under each choice of kernels (PQTopK, batch 1)", "value": best, "unit": "us/step (K = 10, best variant)",
                      "n_gpus": 1, "steps": args.steps, "higher_is_better": False, "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: N={N} d={d} m={m} b={b} batch=1, K in (1, 10, 31)"}, "variants": rows}))


def kcost_mode(args):
    """What K costs on --config at --batch: for K in 1, 10, 100, 512 the scan kernel alone (HIP events around back-to-back
    launches) and the whole pq_score_topk call (scan + fold, enqueued back to back), each result compared with the oracle
    (all queries of the batch up to 8)."""
    import numpy as np
    import torch
    from oracle import pq_oracle
    from paper_2408_09992_amd import binding as pq, workloads as W

    cfg = W.CONFIGS[args.config]
    B = args.batch if args.batch is not None else cfg.batches[0]
    G, cent, Q = W.make(cfg, B=B)
    N, m, b, d = cfg.N, cfg.m, cfg.b, cfg.d
    Gd, Cd, Qd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
    sub = pq.PreparedSubitemScores(Qd, Cd)
    sub()
    torch.cuda.synchronize()
    S_host = sub.S.cpu().numpy()
    rows = []
    for K in (1, 10, 100, 512):
        top = pq.PreparedScoreTopK(Gd, sub.S, K)
        iters = int(max(5, min(1000, 2e8 / (float(N) * B))))
        t_warm = time.perf_counter()
        while time.perf_counter() - t_warm < 0.03:
            for _ in range(iters):
                top()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        calls = []
        for _ in range(5):
            e0.record()
            for _ in range(iters):
                top()
            e1.record()
            torch.cuda.synchronize()
            calls.append(e0.elapsed_time(e1) / iters * 1e3)
        n_prof = max(3, min(50, iters))
        scan_us = sorted(pq.pq_score_topk_profile(Gd, sub.S, K, n_prof, workspace=top.workspace) for _ in range(5))[2] * 1e3
        nq = min(B, 8)
        rid, rsc = pq_oracle.score_topk(G, S_host[:nq], K)
        parity = bool(np.array_equal(top.ids.cpu().numpy()[:nq], rid) and
                      np.array_equal(top.scores.cpu().numpy()[:nq].view(np.uint32), rsc.view(np.uint32)))
        rows.append({"K": K, "scan_kernel_us": scan_us, "pq_score_topk_us": sorted(calls)[2], "parity_vs_oracle": parity})
        print(f"{cfg.name} B={B} K={K:3d}  scan {scan_us:9.2f} us  scan + fold {sorted(calls)[2]:9.2f} us  parity {parity}",
              file=sys.stderr, flush=True)
    print(json.dumps({"metric": "cost of K: scan kernel and pq_score_topk call", "value": rows[1]["pq_score_topk_us"], "unit": "us (K = 10)",
                      "n_gpus": 1, "higher_is_better": False, "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: N={N} d={d} m={m} b={b} batch={B}, K in (1, 10, 100, 512)"}, "kcost": rows}))


def matrix_cores_mode(args):
    """The two dense contractions beside the scan, on the matrix cores and on the scalar kernels
    (pq_measure_force_general bit 2): Eq. 4 over batch sizes (chains of K = 1 fp32 matrix instructions, bit-equal to the
    fused chain: checked against the oracle), and the default scorer W phi (Eq. 3) for batches on the headline catalogue
    (2.62 GB embedding matrix read once per batch instead of once per query)."""
    import numpy as np
    import torch
    from oracle import pq_oracle
    from paper_2408_09992_amd import binding as pq, workloads as W

    cfg = W.CONFIGS[args.config]
    N, m, b, d = cfg.N, cfg.m, cfg.b, cfg.d
    G, cent, Q = W.make(cfg, B=4096)
    Gd, Cd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda()

    def timed(fn, n):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t = []
        for _ in range(3):
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            t.append(e0.elapsed_time(e1) / n * 1e3)
        return sorted(t)[1]

    eq4, default = [], []
    try:
        for B in (1, 64, 256, 448, 1024, 4096):
            Qd = torch.from_numpy(np.ascontiguousarray(Q[:B])).cuda()
            sub = pq.PreparedSubitemScores(Qd, Cd)
            res = {}
            for mask in (4, 0):
                pq.pq_measure_force_general(mask)
                for _ in range(300):
                    sub()
                res[mask] = timed(sub, 500)
            pq.pq_measure_force_general(0)
            sub()
            torch.cuda.synchronize()
            ref = pq_oracle.subitem_scores(np.ascontiguousarray(Q[:B]), cent)
            ok = bool(np.array_equal(sub.S.cpu().numpy().view(np.uint32), ref.view(np.uint32)))
            eq4.append({"B": B, "scalar_kernels_us": res[4], "library_choice_us": res[0], "bit_equal_to_oracle": ok})
            print(f"Eq. 4  B={B:5d}: scalar kernels {res[4]:7.2f} us   library's choice {res[0]:7.2f} us   bit-equal to the oracle {ok}",
                  file=sys.stderr, flush=True)
        Wd = pq.pq_reconstruct_items(Gd, Cd)
        for B in (1, 2, 4, 16, 64, 128):
            Qd = torch.from_numpy(np.ascontiguousarray(Q[:B])).cuda()
            out = torch.empty((B, N), dtype=torch.float32, device="cuda")
            res = {}
            for mask in (4, 0):
                pq.pq_measure_force_general(mask)
                res[mask] = timed(lambda: pq.pq_default_scores(Wd, Qd, out=out), 3 if (mask == 4 and B > 4) else 10)
                if mask == 4:
                    ref = out.clone()
            pq.pq_measure_force_general(0)
            err = float((out - ref).abs().max())
            default.append({"B": B, "matvec_per_query_us": res[4], "library_choice_us": res[0], "TFLOPs": 2.0 * N * d * B / res[0] / 1e6,
                            "W_read_TBps": N * d * 4 / res[0] / 1e6, "max_abs_diff_between_paths": err})
            print(f"Eq. 3  B={B:4d}: mat-vec per query {res[4]:9.1f} us   library's choice {res[0]:9.1f} us "
                  f"({2.0 * N * d * B / res[0] / 1e6:6.1f} TFLOP/s, W at {N * d * 4 / res[0] / 1e6:5.2f} TB/s)   max |diff| {err:.2e}",
                  file=sys.stderr, flush=True)
    finally:
        pq.pq_measure_force_general(0)
    print(json.dumps({"metric": "Eq. 4 and the default scorer on the matrix cores against the scalar kernels", "value": eq4[-2]["library_choice_us"],
                      "unit": "us (Eq. 4, B = 1024)", "n_gpus": 1, "higher_is_better": False, "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": f"{cfg.name}: N={N} d={d} m={m} b={b}; Eq. 4 at B = 1 .. 4096, Eq. 3 at B = 1 .. 128"},
                      "eq4": eq4, "default_scorer": default}))


def breakdown_mode(args):
    """Where the time of a step goes: the three launches of a single-query step (Eq. 4, scan, fold) are run with the
    kernels' stamping instances (wall-clock stamps at fixed points, lane 0 of every wave), back to back as in the timed
    loop, and the last step's stamps are read; repeated --breakdown-samples times, medians over samples.  Times are
    microseconds after the first wave of the Eq. 4 kernel started, unless noted."""
    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W

    cfg = W.CONFIGS[args.config]
    B = args.batch if args.batch is not None else 1
    G, cent, Q = W.make(cfg, B=B)
    N, m, b, K, d = cfg.N, cfg.m, cfg.b, cfg.K, cfg.d
    Gd, Cd, Qd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
    S = torch.empty((B, m, b), dtype=torch.float32, device="cuda")
    ws = torch.empty(pq.pq_score_topk_workspace_bytes(N, B, m, b, K), dtype=torch.uint8, device="cuda")
    ids = torch.empty((B, K), dtype=torch.int32, device="cuda")
    sc = torch.empty((B, K), dtype=torch.float32, device="cuda")
    stamps = torch.zeros((3, pq.PQ_STAMP_RECORDS, pq.PQ_STAMP_SLOTS), dtype=torch.int64, device="cuda")
    tick_us = 0.01                                           # wall_clock64(): 100 MHz on MI355X
    names = {0: "entry", 1: "requested", 2: "tables", 3: "codes", 4: "scored", 5: "offered", 6: "streamed", 7: "selected",
             8: "end", 9: "loaded", 10: "cut", 11: "collected"}
    rows = []
    for _ in range(args.breakdown_samples):
        for _ in range(args.breakdown_steps):
            nblk, waves = pq.pq_measure_step_stamps(Qd, Cd, Gd, K, S, ids, sc, ws, stamps)
        torch.cuda.synchronize()
        t = stamps.cpu().numpy().astype(np.float64)
        eq4 = t[0][t[0][:, 0] > 0]
        scan = t[1][: nblk * waves]
        fold = t[2][t[2][:, 0] > 0]
        if len(eq4):
            t0 = eq4[:, 0].min()
            row = {"eq4_first_entry": 0.0, "eq4_last_end": (eq4[:, 8].max() - t0) * tick_us}
        else:                                                # (no stamping instance of Eq. 4 for this shape: times count from the scan's first wave)
            t0 = scan[:, 0][scan[:, 0] > 0].min()
            row = {}
        for slot in (0, 1, 2, 3, 4, 5, 6, 7, 8):
            col = scan[:, slot]
            col = col[col > 0]
            if len(col):
                row[f"scan_{names[slot]}_first"] = (col.min() - t0) * tick_us
                row[f"scan_{names[slot]}_median"] = (np.median(col) - t0) * tick_us
                row[f"scan_{names[slot]}_last"] = (col.max() - t0) * tick_us
        for (s0, s1) in ((0, 2), (2, 3), (3, 4), (2, 4), (4, 5), (5, 6), (5, 7), (6, 7), (7, 8)):   # per-wave durations
            ok = (scan[:, s0] > 0) & (scan[:, s1] > 0)
            if ok.any():
                dd = (scan[ok, s1] - scan[ok, s0]) * tick_us
                row[f"scan_wave_{names.get(s0, s0)}_to_{names.get(s1, s1)}_median"] = float(np.median(dd))
                row[f"scan_wave_{names.get(s0, s0)}_to_{names.get(s1, s1)}_max"] = float(dd.max())
        for slot in (0, 9, 10, 11, 5, 7, 8):
            col = fold[:, slot]
            col = col[col > 0]
            if len(col):
                row[f"fold_{names[slot]}_first"] = (col.min() - t0) * tick_us
                row[f"fold_{names[slot]}_last"] = (col.max() - t0) * tick_us
        rows.append(row)
        stamps.zero_()
    keys = list(rows[0].keys())
    med = {k: float(np.median([r[k] for r in rows if k in r])) for k in keys}
    for k in keys:
        print(f"{k:28s} {med[k]:8.2f} us", file=sys.stderr)
    print(json.dumps({
        "metric": "in-kernel wall-clock stamps of one step (Eq. 4, scan, fold), microseconds after the step's first wave",
        "value": med["fold_end_last"], "unit": "us", "n_gpus": 1, "higher_is_better": False, "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N} d={d} m={m} b={b} K={K} batch={B}, codes {cfg.codes}, seed {cfg.seed}",
                   "scan_workgroups": nblk, "waves_per_workgroup": waves, "samples": args.breakdown_samples,
                   "steps_per_sample": args.breakdown_steps, "tick_us": tick_us},
        "stamps_us": med}))


def yardsticks_mode(args):
    """What this machine gives: the cost of an empty launch, a plain streaming read of 10 MB and 400 MB, and random
    gathers from LDS (4-, 8- and 16-byte words, 8 KB and 32 KB tables, 8 and 16 waves per CU) against the conflict-free
    case.  These are the denominators the scan kernels' figures are held to."""
    import torch
    from paper_2408_09992_amd import binding as pq

    props = torch.cuda.get_device_properties(0)
    cus = props.multi_processor_count
    out = {"compute_units": cus, "nominal_clock_GHz": 2.4}
    for _ in range(3):
        pq.pq_measure_empty_launch(256, 512, 500)
    out["empty_launch_us"] = {f"{blocks}x{threads}": sorted(pq.pq_measure_empty_launch(blocks, threads, 1000) for _ in range(5))[2] * 1e3
                              for (blocks, threads) in ((1, 64), (256, 512), (512, 512), (256, 1024))}
    reads = {}
    for nbytes in (10_240_000, 400_000_000):
        buf = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        pq.pq_read_bandwidth_profile(buf, 20)
        ms = sorted(pq.pq_read_bandwidth_profile(buf, 50) for _ in range(5))[2]
        reads[str(nbytes)] = {"us": ms * 1e3, "GBps": nbytes / (ms * 1e-3) / 1e9}
        del buf
    out["stream_read"] = reads
    # synchronising inside a launch against a launch boundary (why a step stays three launches)
    scratch = torch.zeros(pq.PQ_SYNC_SCRATCH_BYTES, dtype=torch.uint8, device="cuda")
    sync = {}
    for v, name in enumerate(pq.PQ_SYNC_VARIANT_NAMES):
        pq.pq_measure_sync_variant(v, scratch, 200)
        sync[name] = sorted(pq.pq_measure_sync_variant(v, scratch, 1000) for _ in range(5))[2] * 1e3
        print(f"sync variant {name:28s} {sync[name]:7.2f} us per iteration", file=sys.stderr, flush=True)
    out["in_launch_sync_us"] = sync
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    gathers = []
    rounds = 16 * 256
    for width in (4, 8, 16):
        for table in (8192, 32768):
            for threads, blocks_per_cu in ((512, 1), (1024, 1), (512, 2)):
                for cf in (False, True):
                    blocks = cus * blocks_per_cu
                    pq.pq_measure_lds_gather(width, table, rounds, cf, blocks, threads, 3, sink)
                    ms = sorted(pq.pq_measure_lds_gather(width, table, rounds, cf, blocks, threads, 10, sink) for _ in range(5))[2]
                    lane_reads = blocks * threads * rounds
                    per_ns = lane_reads / (ms * 1e6)
                    g = {"width": width, "table_bytes": table, "threads": threads, "workgroups_per_cu": blocks_per_cu,
                         "conflict_free": cf, "us": ms * 1e3, "lane_reads_per_ns": per_ns,
                         "lane_reads_per_clk_per_cu": per_ns / 2.4 / cus, "GBps": per_ns * width,
                         "bytes_per_clk_per_cu": per_ns * width / 2.4 / cus}
                    gathers.append(g)
                    print(f"lds gather w={width:2d} table={table:6d} {threads:4d}x{blocks_per_cu} {'conflict-free' if cf else 'random       '} "
                          f"{ms * 1e3:8.1f} us  {g['lane_reads_per_clk_per_cu']:6.2f} lane reads/clk/CU  {g['bytes_per_clk_per_cu']:6.1f} B/clk/CU  "
                          f"{g['GBps'] / 1e3:6.1f} TB/s", file=sys.stderr, flush=True)
    # replicated tables (the scan's layout for one query): 2048 entries of 4 bytes, C copies side by side
    for copies in (1, 2, 4, 8, 16):
        for threads, blocks_per_cu in ((512, 1), (1024, 1)):
            table, blocks = 8192 * copies, cus * blocks_per_cu
            pq.pq_measure_lds_gather(4, table, rounds, False, blocks, threads, 3, sink, copies=copies)
            ms = sorted(pq.pq_measure_lds_gather(4, table, rounds, False, blocks, threads, 10, sink, copies=copies) for _ in range(5))[2]
            per_ns = blocks * threads * rounds / (ms * 1e6)
            g = {"width": 4, "table_bytes": table, "copies": copies, "threads": threads, "workgroups_per_cu": blocks_per_cu,
                 "conflict_free": False, "us": ms * 1e3, "lane_reads_per_ns": per_ns,
                 "lane_reads_per_clk_per_cu": per_ns / 2.4 / cus, "GBps": per_ns * 4, "bytes_per_clk_per_cu": per_ns * 4 / 2.4 / cus}
            gathers.append(g)
            print(f"lds gather w= 4 entries=2048 copies={copies:2d} {threads:4d}x{blocks_per_cu} random  {ms * 1e3:8.1f} us  "
                  f"{g['lane_reads_per_clk_per_cu']:6.2f} lane reads/clk/CU", file=sys.stderr, flush=True)
    out["lds_gather"] = gathers
    best16 = max(g["GBps"] for g in gathers if g["width"] == 16 and not g["conflict_free"])
    print(json.dumps({"metric": "machine yardsticks (empty launch, streaming read, random LDS gathers)", "value": best16,
                      "unit": "GB/s (random 16-byte LDS gathers, best configuration)", "n_gpus": 1, "higher_is_better": True,
                      "vs_baseline": None, "dtype": "u32", "data": "synthetic",
                      "config": {"workload": "yardsticks: no catalogue; hashed offsets into an LDS table"}, "yardsticks": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # (the GPU needs some 20 ms of continuous work after idling before its clocks settle: the default warm-up is long
    # enough for that on every workload, and still only a fraction of a second)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--config", default="large")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-iters", type=int, default=50)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of the code matrix (N*m bytes read, N*m written): "
                         "the known-size kernel that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--sweep", action="store_true", help="catalogue-size sweep (m = 8 and 64, N = 10^3 .. 10^9) "
                    "instead of one workload; per-point lines on stderr, one JSON line on stdout")
    ap.add_argument("--compare", action="store_true", help="time PQTopK against the paper's two other scorers "
                    "(Algorithm 2 and the default matrix-vector product) on --config at batch 1")
    ap.add_argument("--subset", action="store_true", help="time candidate-list scoring (pq_score_topk_subset) over "
                    "list sizes on --config at batch 1")
    ap.add_argument("--wide", action="store_true", help="time codebooks with 16-bit sub-ids (pq_score_topk_u16) over "
                    "alphabet and catalogue sizes at batch 1")
    ap.add_argument("--breakdown", action="store_true", help="in-kernel wall-clock stamps of the three launches of one "
                    "single-query step on --config (m = 8 only)")
    ap.add_argument("--breakdown-samples", type=int, default=20)
    ap.add_argument("--breakdown-steps", type=int, default=50)
    ap.add_argument("--variants", action="store_true", help="step time of --config at batch 1 with the short scan / small fold "
                    "and with the general kernels in their place")
    ap.add_argument("--kcost", action="store_true", help="scan kernel and pq_score_topk call for K = 1, 10, 100, 512 on --config "
                    "at --batch")
    ap.add_argument("--matrix-cores", action="store_true", help="Eq. 4 and the default scorer (Eq. 3) on the matrix cores "
                    "against the scalar kernels, over batch sizes")
    ap.add_argument("--yardsticks", action="store_true", help="machine yardsticks: empty launch, plain streaming read, "
                    "random gathers from LDS")
    ap.add_argument("--sweep-max-bytes", type=float, default=7e10, help="largest code matrix the sweep allocates")
    ap.add_argument("--sweep-check-bytes", type=float, default=1e9,
                    help="largest code matrix whose result the sweep checks against the oracle")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.sweep:
        sweep(args)
        return
    if args.compare:
        compare(args)
        return
    if args.subset:
        subset_mode(args)
        return
    if args.wide:
        wide_mode(args)
        return
    if args.breakdown:
        breakdown_mode(args)
        return
    if args.yardsticks:
        yardsticks_mode(args)
        return
    if args.variants:
        variants_mode(args)
        return
    if args.kcost:
        kcost_mode(args)
        return
    if args.matrix_cores:
        matrix_cores_mode(args)
        return

    import numpy as np
    import torch
    from paper_2408_09992_amd import binding as pq, workloads as W

    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU")
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    B = args.batch if args.batch is not None else cfg.batches[0]
    G, cent, Q = W.make(cfg, B=B)
    N, m, b, K, d = cfg.N, cfg.m, cfg.b, cfg.K, cfg.d

    Gd, Cd, Qd = torch.from_numpy(G).cuda(), torch.from_numpy(cent).cuda(), torch.from_numpy(Q).cuda()
    Sd = torch.empty((B, m, b), dtype=torch.float32, device="cuda")
    ws = torch.empty(pq.pq_score_topk_workspace_bytes(N, B, m, b, K), dtype=torch.uint8, device="cuda")
    ids = torch.empty((B, K), dtype=torch.int32, device="cuda")
    sc = torch.empty((B, K), dtype=torch.float32, device="cuda")

    sub = pq.PreparedSubitemScores(Qd, Cd, out=Sd)
    top = pq.PreparedScoreTopK(Gd, Sd, K, workspace=ws, out_ids=ids, out_scores=sc)

    def step():
        sub()
        top()

    if args.calibrate_copy:
        torch.empty_like(Gd).copy_(Gd)
        torch.cuda.synchronize()

    t_warm = time.perf_counter()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warmup_run = args.warmup
    while time.perf_counter() - t_warm < 0.03:             # (untimed) a GPU that was idle needs ~20 ms of work before
        for _ in range(50):                                 # its clocks settle, however few warm-up steps were asked for
            step()
        warmup_run += 50                                    # (reported: `warmup_steps_run`)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    el = time.perf_counter() - t0

    # parity of the timed run's own output, against the oracle
    from oracle import pq_oracle
    # (every query of the batch up to 128; of a larger batch 128 spread evenly, the first and the last among them)
    checked = np.arange(B) if B <= 128 else np.unique(np.linspace(0, B - 1, 128).round().astype(np.int64))
    rid, rsc = pq_oracle.pqtopk(G, cent, np.ascontiguousarray(Q[checked]), K)
    got_ids, got_sc = ids.cpu().numpy()[checked], sc.cpu().numpy()[checked]
    parity = bool(np.array_equal(got_ids, rid) and np.all(np.abs(got_sc - rsc) <= 1e-5 * np.maximum(np.abs(rsc), 1.0)))

    # the scan kernel's own duration: median of five back-to-back sequences.  The oracle run above left the GPU idle
    # for tens of milliseconds, so its clocks are brought back up first (untimed).
    t_warm = time.perf_counter()
    while time.perf_counter() - t_warm < 0.04:
        pq.pq_score_topk_profile(Gd, Sd, K, args.profile_iters, workspace=ws)
    scan_ms = sorted(pq.pq_score_topk_profile(Gd, Sd, K, args.profile_iters, workspace=ws) for _ in range(5))[2]
    torch.cuda.synchronize()
    algo_bytes = float(N) * m                               # one pass over the code matrix per launch
    achieved = algo_bytes / (scan_ms * 1e-3) / 1e9

    # what a kernel that only reads gets out of this machine on the same bytes: the yardstick beside the published peak
    pq.pq_read_bandwidth_profile(Gd, args.profile_iters)
    read_ms = sorted(pq.pq_read_bandwidth_profile(Gd, args.profile_iters) for _ in range(5))[2]
    read_gbs = algo_bytes / (read_ms * 1e-3) / 1e9
    # ... and on 16 bytes: what one launch costs on this machine when it has nothing to do (back-to-back launches)
    tiny = Gd.view(-1)[:16]
    pq.pq_read_bandwidth_profile(tiny, 200)
    floor_us = sorted(pq.pq_read_bandwidth_profile(tiny, 200) for _ in range(5))[2] * 1e3

    # stage times (HIP events on the stream the kernels run on, back-to-back launches of one stage)
    def stage_us(fn, iters=200):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3
    n_stage = 200 if N * B < 2e8 else 20
    t_sub, t_top = stage_us(sub, n_stage), stage_us(top, n_stage)

    # one call at a time (the paper's per-user response time: Table 3 quotes a median, Figure 2 a mean): host-side
    # time from enqueue to completion of one step, caches warm; then the same with the caches evicted before every call
    lat = []
    for _ in range(200 if N * B < 2e8 else 30):
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        lat.append((time.perf_counter() - t1) * 1e6)
    lat = np.asarray(lat)
    evict = torch.empty(768 << 20, dtype=torch.uint8, device="cuda")       # larger than L2 + the 256 MB Infinity Cache
    cold = []
    for i in range(20):
        evict.fill_(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        cold.append((time.perf_counter() - t1) * 1e6)
    cold = np.asarray(cold)
    del evict

    ms_per_step = el / args.steps * 1e3
    workload = f"{cfg.name}: N={N} d={d} m={m} b={b} K={K} batch={B}, codes {cfg.codes}, seed {cfg.seed}"
    traffic, traffic_source = measured_traffic(workload)
    out = {
        "metric": "items scored/sec (PQTopK, whole path incl. top-K)",
        "value": N * B * args.steps / el,
        "unit": "items/s",
        "queries_per_s": B * args.steps / el,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "warmup_steps_run": warmup_run, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload},
        "parity_vs_oracle": parity, "parity_queries_checked": int(len(checked)),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "catalogue scan (Eq. 5 + per-workgroup top-K)", "kernel_ms": scan_ms,
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "read_kernel_GBps": read_gbs, "frac_of_read_kernel": achieved / read_gbs,
                     "empty_launch_us": floor_us},
        "stage_us": {"pq_subitem_scores": t_sub, "pq_score_topk": t_top, "scan_kernel": scan_ms * 1e3},
        # the whole step against the HBM peak: codes once, S written and read, results written, over the step time
        "whole_step": {"effective_GBps": (algo_bytes + 4.0 * B * m * b + 8.0 * B * K) / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": (algo_bytes + 4.0 * B * m * b + 8.0 * B * K) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "latency_us": {"what": "one step at a time, host enqueue to completion", "median": float(np.median(lat)),
                       "mean": float(lat.mean()), "p99": float(np.percentile(lat, 99)),
                       "cold_caches_median": float(np.median(cold))},
    }
    if B > 1:
        # a batch re-uses every code byte B times: the table lookups (4 bytes gathered from LDS per split, item and
        # query), not HBM, bound the scan; reported beside the HBM figure, against what the LDS returns at best on paper
        # (`peak`: 128 bytes per clock and CU) and against what random 16-byte gathers get out of it on this machine,
        # measured by this run (`measured_peak`; the batched kernel reads four queries' values with one such gather)
        lds_bytes = 4.0 * m * N * B
        lds_achieved = lds_bytes / (scan_ms * 1e-3) / 1e9
        lds_measured = measured_lds_peak(pq, torch)
        out["lds_gather"] = {"bound": "lds", "achieved": lds_achieved, "peak": LDS_PEAK_GBS,
                             "unit": "GB/s", "frac": lds_achieved / LDS_PEAK_GBS,
                             "measured_peak": lds_measured, "frac_of_measured": lds_achieved / lds_measured,
                             "measured_peak_what": "random 16-byte gathers from a 32 KB LDS table, 16 waves per CU, nothing else (pq_measure_lds_gather)",
                             "algorithmic_bytes_per_launch": lds_bytes}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(G, cent, Q, K)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
