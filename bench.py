"""Benchmark of the GNN-Descent k-NN graph build on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2] [--n N]

One "step" is one whole build (norms, random lists, it1 phase-1 rounds, it2 phase-2 rounds,
finalize) of the 1M x 128 fp32, k = 32 workload (synthetic stand-in for SIFT-1M) with the
vectors already resident in HBM.  Prints ONE JSON line: points/s at recall@32 >= 0.95, the
local join's fraction of the fp32 MFMA peak (timed with HIP events on the launch stream), and
the CPU oracle timed on a bounded sample of the same workload.
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

MFMA_FP32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0


BENCH_ITERS = 4


def bench_params(k: int, seed: int = 1):
    """The configuration the headline number is quoted on: what the plain entry point runs with,
    tg_knn_build(X, n, d, k, metric, iters = 4, seed, ...): the library's defaults and the smallest round budget
    that reaches recall@32 >= 0.95 on the 1M x 128 workload (four rounds of the first phase)."""
    from paper_2508_08744_amd import knn
    return knn.default_params(k, BENCH_ITERS, seed=seed)


def cpu_baseline(config: str, prm, sample_n: int):
    """The oracle as it stands, one thread, on a bounded sample of the same generator: the plain method
    (its reference mode) is what is timed.  The same sample is built on the GPU and compared with the
    oracle's model of the build's hand-over (ids and distances, bit for bit where the data is integer valued)
    and, for recall, with the plain method at equal rounds."""
    import numpy as np
    import torch
    import oracle
    from paper_2508_08744_amd import inputs, knn
    X = inputs.make(config, n=sample_n)
    plain = oracle.NNDescent(X, prm.k, metric=prm.metric, S=prm.S, R=prm.R, m=prm.m, seed=int(prm.seed))
    t0 = time.perf_counter()
    plain.run(prm.it1, prm.it2)
    dt = time.perf_counter() - t0
    model = oracle.NNDescent(X, prm.k, metric=prm.metric, **oracle.device_model(prm))
    model.run(prm.it1, prm.it2)
    Xg = torch.from_numpy(X).cuda()
    ids, dist, _ = knn.knn_build_ex(Xg, prm)
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    mi, md, _ = model.graph()
    rows = inputs.sample_rows(sample_n, min(10000, sample_n), seed=4)
    truth, _ = knn.exact_knn(Xg, prm.k, inputs.CONFIGS[config]["metric"], torch.from_numpy(rows).cuda())
    truth = truth.cpu().numpy()
    r_gpu, r_plain = oracle.recall(ids[rows], truth), oracle.recall(plain.graph()[0][rows], truth)
    return {"value": sample_n / dt, "unit": "points/s", "cores": 1, "kind": "oracle",
            "sample": "%s generator, n=%d of %d points, same k and round counts, whole build by the plain method, %.1f s"
                      % (config, sample_n, inputs.CONFIGS[config]["n"], dt),
            "identical": bool((ids == mi).all() and (dist.astype(np.float64) == md).all()),
            "recall_gpu": r_gpu, "recall_plain": r_plain, "recall_gap_vs_plain": r_gpu - r_plain}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--n", type=int, default=None, help="override the number of points (debugging)")
    ap.add_argument("--it1", type=int, default=None, help="phase-1 rounds (default: the headline setting)")
    ap.add_argument("--it2", type=int, default=None, help="phase-2 rounds (default: the headline setting)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the build: no pruning and sharding legs (for profiles)")
    ap.add_argument("--cpu-sample", type=int, default=50000)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU; run with --gpus 1 (the method would shard by node range, "
              "but no multi-GPU path is built)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import oracle
    from paper_2508_08744_amd import inputs, knn

    cfg = inputs.CONFIGS[args.config]
    n = args.n or cfg["n"]
    d, k, metric = cfg["d"], cfg["k"], cfg["metric"]
    dev = torch.device("cuda:0")
    big = n > 20_000_000          # the 1e8-point configuration: drawn on the device, rounds in eight parts and 64 slots per node so that it fits
    if big:
        X = None
        Xg = inputs.make_on_device(args.config, dev, n=n)
    else:
        X = inputs.make(args.config, n=n)
        Xg = torch.from_numpy(X).to(dev)
    prm = bench_params(k)
    if big:
        prm.parts, prm.C = 8, 64
    if args.it1 is not None:
        prm.it1 = args.it1
    if args.it2 is not None:
        prm.it2 = args.it2
    prm.metric = knn.METRICS[metric]
    workspace = torch.empty(knn.workspace_bytes(n, d, prm), dtype=torch.uint8, device=dev)

    for _ in range(args.warmup):
        knn.knn_build_ex(Xg, prm, workspace, want_stats=False)
    torch.cuda.synchronize()
    stats = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ids, dist, st = knn.knn_build_ex(Xg, prm, workspace, want_stats=True)
        stats.append(st)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # recall@k on a fixed sample of rows, ground truth by exhaustive search (outside the timed region)
    rows = inputs.sample_rows(n, 10000, seed=4)
    rows_g = torch.from_numpy(rows).to(dev)
    truth, _ = knn.exact_knn(Xg, k, metric, rows_g)
    recall = oracle.recall(ids[rows_g].cpu().numpy(), truth.cpu().numpy())

    # dominant kernel: the phase-1 local join (the kernels that multiply).  Algorithmic flops = 2 d per needed pair
    # (new-new and new-old pairs of every block); duration from the HIP events the library
    # records on the launch stream around each join launch.
    r1 = stats[0]["rounds_phase1"]
    join_ms = [sum(s["ms_join"][:r1]) for s in stats]
    join_flops = [2.0 * d * sum(s["join_pairs"][:r1]) for s in stats]
    launches = r1 * len(stats)
    avg_launch_ms = sum(join_ms) / max(launches, 1)
    achieved = (sum(join_flops) / max(launches, 1)) / (avg_launch_ms * 1e-3) / 1e12 if avg_launch_ms > 0 else 0.0
    gather_gbs = (4.0 * d * sum(sum(s["join_vectors"][:r1]) for s in stats) / max(launches, 1)) / (avg_launch_ms * 1e-3) / 1e9 \
        if avg_launch_ms > 0 else 0.0
    last = stats[-1]
    # HBM bytes per join launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs kept under profiles/ (calibrated
    # against a plain copy); only quoted for the workload those runs were made on
    traffic, traffic_source = None, None
    extras = not big and not args.no_extras      # the pruning and sharding legs below are sized for the headline workload
    tfile = os.path.join(ROOT, "profiles", "join_C2_1Mx128_k32_hbm_traffic.txt")
    if args.config == "C2" and n == cfg["n"] and os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("join_traffic_bytes_per_launch"):
                traffic, traffic_source = float(line.split("=")[1].split()[0]), "profiles/" + os.path.basename(tfile)
    out = {
        "metric": "k-NN graph build points/sec at recall@32>=0.95 (1Mx128 fp32); join MFMA %",
        "value": n / (ms_per_step * 1e-3),
        "unit": "points/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: n=%d d=%d k=%d %s, Gaussian mixture (%s stand-in)" % (
            args.config, n, d, k, metric, {"C1": "small test", "C2": "SIFT-1M", "C3": "Gist", "C4": "Deep", "C5": "Deep"}.get(args.config, "synthetic")),
                   "it1": prm.it1, "it2": prm.it2, "S": prm.S, "R": prm.R, "C": prm.C,
                   "parts": prm.parts, "m": prm.m, "seed": int(prm.seed)},
        "recall_at_k": recall,
        "recall_ok": bool(recall >= 0.95),
        "join_mfma_pct": 100.0 * achieved / MFMA_FP32_PEAK_TFLOPS,
        "roofline": {"bound": "mfma", "kernel": "phase-1 local join of one round (join_wave_kernel<3>, <4> and join_kernel of every part; adj_kernel, which runs before them, is timed apart)",
                     "achieved": achieved,
                     "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_FP32_PEAK_TFLOPS,
                     "avg_launch_ms": avg_launch_ms, "launches": launches, "gather_GBps": gather_gbs,
                     "hbm_gather_frac": gather_gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source},
        "breakdown_ms": {"norms": last["ms_norms"], "init": last["ms_init"], "finalize": last["ms_finalize"],
                         "sample": sum(last["ms_sample"]), "adjacency": sum(last["ms_adjacency"]), "join": sum(last["ms_join"][:r1]),
                         "update": sum(last["ms_update"]), "phase2": sum(last["ms_join"][r1:])},
        "updates_per_round": last["updates"],
    }
    # the plain entry point with the same budget (it takes and returns its workspace in stream order): same graph
    if args.it1 is None and args.it2 is None and not big:
        knn.knn_build(Xg, k, metric, iters=BENCH_ITERS, seed=int(prm.seed))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ids_p, dist_p = knn.knn_build(Xg, k, metric, iters=BENCH_ITERS, seed=int(prm.seed))
        torch.cuda.synchronize()
        ms_p = 1e3 * (time.perf_counter() - t0) / args.steps
        out["tg_knn_build"] = {"iters": BENCH_ITERS, "ms_per_step": ms_p, "points_per_s": n / (ms_p * 1e-3),
                               "identical_to_timed_build": bool((ids_p == ids).all() and (dist_p == dist).all())}
        del ids_p, dist_p
    if not extras:
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(args.config, prm, min(args.cpu_sample, n))
        print(json.dumps(out))
        return
    # the same build with the local join on the fp16 matrix instructions where that is exact (join_f16 = 2: the library
    # checks on the device that every value is an fp16 number, as byte-valued features are; off by default and not part
    # of `value`): the graph must come out bit for bit the same
    if args.config == "C2" and n == cfg["n"]:
        prm16 = bench_params(k)
        prm16.metric = prm.metric
        prm16.it1, prm16.it2, prm16.join_f16 = prm.it1, prm.it2, 2
        ws16 = torch.empty(knn.workspace_bytes(n, d, prm16), dtype=torch.uint8, device=dev)
        knn.knn_build_ex(Xg, prm16, ws16, want_stats=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            ids16, dist16, st16 = knn.knn_build_ex(Xg, prm16, ws16, want_stats=True)
        torch.cuda.synchronize()
        ms16 = 1e3 * (time.perf_counter() - t0) / 3
        r16 = st16["rounds_phase1"]
        out["join_f16"] = {"ms_per_step": ms16, "points_per_s": n / (ms16 * 1e-3), "ms_join": sum(st16["ms_join"][:r16]),
                           "join_launch_ms": sum(st16["ms_join"][:r16]) / max(r16, 1),
                           "recall_at_k": oracle.recall(ids16[rows_g].cpu().numpy(), truth.cpu().numpy()),
                           "identical_to_fp32_join": bool((ids16 == ids).all() and (dist16 == dist).all())}
        del ws16, ids16, dist16
    # the next step after the hot path: rank-based pruning of the graph just built (outside `value`).
    # Algorithmic bytes per node: its row, the entries in front of every neighbour's own position, the output.
    d_out = k // 2
    pr_ms = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        pruned = knn.prune_rank(ids, d_out)
        e1.record()
        torch.cuda.synchronize()
        pr_ms.append(e0.elapsed_time(e1))
    pr_ms = sorted(pr_ms)[len(pr_ms) // 2]
    pr_bytes = n * (4.0 * k + 2.0 * k * (k - 1) + 4.0 * d_out)
    out["prune_rank"] = {"k": k, "d_out": d_out, "ms": pr_ms, "points_per_s": n / (pr_ms * 1e-3),
                         "roofline": {"bound": "hbm", "achieved": pr_bytes / (pr_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                      "unit": "GB/s", "frac": pr_bytes / (pr_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}}
    # and the distance-based pruning (Vamana's rule over the neighbours, NSG's over two hops) and the angle-based
    # one (NSSG's rule at 60 degrees, over the neighbours and over two hops) of the same graph.
    # Algorithmic bytes per node: the rows of its candidates (all k neighbours; over two hops every distinct
    # candidate once, counted on a sample of nodes) and of itself, the id rows read, the output.
    pd_cases = []
    if metric == "l2":
        uniq = ids[:4096].long()
        two = torch.cat([uniq[:, :, None].expand(-1, -1, 1), ids[uniq.reshape(-1)].reshape(4096, k, k).long()], dim=2).reshape(4096, -1)
        two = two.sort(dim=1).values
        q_mean = float(((two[:, 1:] != two[:, :-1]).sum(dim=1) + 1).float().mean())     # distinct ids within two hops (self included)
        for name, rule, hops, thres, cands in (("prune_dist_1hop", "alpha", 1, 1.2, float(k)), ("prune_dist_2hop", "alpha", 2, 1.0, q_mean),
                                               ("prune_angle_1hop", "gamma_deg", 1, 60.0, float(k)),
                                               ("prune_angle_2hop", "gamma_deg", 2, 60.0, q_mean),       # NSSG's setting in the paper
                                               ("prune_dispersion_1hop", "d_out", 1, k // 2, float(k))):  # DPG: half of the neighbours
            ms_l = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                if rule == "alpha":
                    pd_out = knn.prune_dist(Xg, ids, k, alpha=thres, hops=hops)
                elif rule == "gamma_deg":
                    pd_out = knn.prune_angle(Xg, ids, k, gamma_deg=thres, hops=hops)
                else:
                    pd_out = knn.prune_dispersion(Xg, ids, thres, hops=hops)
                e1.record()
                torch.cuda.synchronize()
                ms_l.append(e0.elapsed_time(e1))
            ms_pd = sorted(ms_l)[len(ms_l) // 2]
            by = n * (4.0 * d * (cands + 1) + 4.0 * k * (1 if hops == 1 else 1 + k) + 4.0 * pd_out.shape[1])
            pd_cases.append((name, rule, hops, thres, pd_out))
            out[name] = {
                rule: thres, "d_out": pd_out.shape[1], "mean_degree": float((pd_out >= 0).sum(dim=1).float().mean()), "cand_size": 64, "candidates_per_node": cands, "ms": ms_pd,
                "points_per_s": n / (ms_pd * 1e-3),
                "roofline": {"bound": "hbm", "achieved": by / (ms_pd * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": by / (ms_pd * 1e-3) / 1e9 / HBM_PEAK_GBS}}
    # the same build with the other two algorithm seeds (the timed region above is seed 1): time and recall of each
    if extras:
        out["other_seeds"] = {}
        for seed in (2, 3):
            prm_s = bench_params(k, seed=seed)
            prm_s.metric, prm_s.it1, prm_s.it2, prm_s.C, prm_s.parts = prm.metric, prm.it1, prm.it2, prm.C, prm.parts
            knn.knn_build_ex(Xg, prm_s, workspace, want_stats=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                ids_s, _, _ = knn.knn_build_ex(Xg, prm_s, workspace, want_stats=False)
            torch.cuda.synchronize()
            ms_s = 1e3 * (time.perf_counter() - t0) / 3
            out["other_seeds"][str(seed)] = {"ms_per_step": ms_s, "points_per_s": n / (ms_s * 1e-3),
                                             "recall_at_k": oracle.recall(ids_s[rows_g].cpu().numpy(), truth.cpu().numpy())}
    # sharded construction (the clusters of the paper's large-scale framework): every point goes to its 2 closest
    # of 8 centres (a few Lloyd steps on a sample: input preparation, untimed), every cluster is built on its own
    # with the same parameters and merged into the global lists.  Merge bytes per local node: its global row read
    # and written, its local row, the translated ids.
    shard_last = None
    if n >= 100000:
        nc, copies = 8, 2
        gen = torch.Generator(device="cpu").manual_seed(2)
        centres = Xg[torch.randperm(n, generator=gen)[:nc].to(dev)].clone()
        samp = Xg[::16]
        for _ in range(5):
            a = torch.cdist(samp, centres).argmin(dim=1)
            for c in range(nc):
                if bool((a == c).any()):
                    centres[c] = samp[a == c].mean(dim=0)
        near = torch.cdist(Xg, centres).topk(copies, dim=1, largest=False).indices
        members = [torch.nonzero((near == c).any(dim=1)).flatten().to(torch.int32) for c in range(nc)]
        Xs = [Xg[mm.long()].contiguous() for mm in members]
        wss = [torch.empty(knn.workspace_bytes(x.shape[0], d, prm), dtype=torch.uint8, device=dev) for x in Xs]
        for rep in range(2):
            g_ids, g_dist = knn.lists_clear(n, k)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * nc + 1)]
            ev[0].record()
            for c in range(nc):
                l_ids, l_dist, _ = knn.knn_build_ex(Xs[c], prm, wss[c], want_stats=False)
                ev[2 * c + 1].record()
                if c == nc - 1:
                    before = (g_ids.clone(), g_dist.clone())
                    ev[2 * c + 1].record()
                knn.merge_local(g_ids, g_dist, l_ids, l_dist, members[c])
                ev[2 * c + 2].record()
            torch.cuda.synchronize()
        ms_b = sum(ev[2 * c].elapsed_time(ev[2 * c + 1]) for c in range(nc))
        ms_m = sum(ev[2 * c + 1].elapsed_time(ev[2 * c + 2]) for c in range(nc))
        shard_last = (before, l_ids, l_dist, members[nc - 1], g_ids, g_dist)
        nl = sum(int(mm.numel()) for mm in members)
        mby = nl * (8.0 * k + 8.0 * k + 8.0 * k + 4.0 * k)
        out["sharded_build"] = {
            "clusters": nc, "copies_per_point": copies, "cluster_sizes": [int(mm.numel()) for mm in members],
            "ms_builds": ms_b, "ms_merges": ms_m, "points_per_s": n / ((ms_b + ms_m) * 1e-3),
            "recall_at_k": oracle.recall(g_ids[rows_g].cpu().numpy(), truth.cpu().numpy()),
            "merge_roofline": {"bound": "hbm", "achieved": mby / (ms_m * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": mby / (ms_m * 1e-3) / 1e9 / HBM_PEAK_GBS}}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, prm, min(args.cpu_sample, n))
        if shard_last is not None:
            (b_ids, b_dist), l_ids, l_dist, mm, a_ids, a_dist = shard_last
            w_ids, w_dist = b_ids.cpu().numpy(), b_dist.cpu().numpy()
            t0 = time.perf_counter()
            oracle.merge_local(w_ids, w_dist, l_ids.cpu().numpy(), l_dist.cpu().numpy(), mm.cpu().numpy())
            dt = time.perf_counter() - t0
            out["sharded_build"]["cpu_baseline"] = {
                "value": int(mm.numel()) / dt, "unit": "merged lists/s", "cores": 1, "kind": "oracle",
                "sample": "the merge of the last cluster (%d nodes) into the lists of the other seven, %.1f s" % (int(mm.numel()), dt),
                "identical": bool((a_ids.cpu().numpy() == w_ids).all() and (a_dist.cpu().numpy() == w_dist).all())}
        ids_h = ids.cpu().numpy()
        for name, rule, hops, thres, pd_out in pd_cases:
            n_do = min(n, 20000 if hops == 1 else 3000)
            t0 = time.perf_counter()
            if rule == "d_out":
                want, _, margin = oracle.filter_dpg(X, ids_h, hops, 64, thres, n_do=n_do)
                tol = 64.0 * (d + 8) * 2.0 ** -24
            elif rule == "alpha":
                want, _, margin = oracle.filter_dist(X, ids_h, hops, 64, thres, k, n_do=n_do)
                tol = 4.0 * (d + 8) * 2.0 ** -24 * max(1.0, thres * thres)
            else:
                want, _, margin = oracle.filter_angle(X, ids_h, hops, 64, thres, k, n_do=n_do)
                tol = 8.0 * (d + 8) * 2.0 ** -24
            dt = time.perf_counter() - t0
            same = (pd_out[:n_do].cpu().numpy() == want).all(axis=1)
            # on data that is not integer valued a row may differ where the oracle says a decision was within
            # fp32 rounding of a tie (its margin for the row is below the tolerance the parity tests use)
            out[name]["cpu_baseline"] = {
                "value": n_do / dt, "unit": "points/s", "cores": 1, "kind": "oracle",
                "sample": "rows of the first %d nodes of the graph just built, %.1f s" % (n_do, dt),
                "identical": bool(same.all()), "rows_identical": float(same.mean()),
                "other_rows_are_near_ties": bool((margin[~same] < tol).all())}
        n_do = min(n, 50000)
        t0 = time.perf_counter()
        want, _ = oracle.prune_rank(ids.cpu().numpy(), d_out, n_do=n_do)
        dt = time.perf_counter() - t0
        out["prune_rank"]["cpu_baseline"] = {"value": n_do / dt, "unit": "points/s", "cores": 1, "kind": "oracle",
                                             "sample": "rows of the first %d nodes of the graph just built, %.1f s" % (n_do, dt),
                                             "identical": bool((pruned[:n_do].cpu().numpy() == want).all())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
