"""The benchmark configuration (1M x 128, k = 32) in the launch configuration bench.py times:
properties that hold at any size, and sampled rows checked one by one against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def test_c2_full_size():
    cfg = inputs.CONFIGS["C2"]
    n, d, k = cfg["n"], cfg["d"], cfg["k"]
    X = inputs.make("C2")
    Xg = torch.from_numpy(X).cuda()
    import bench
    prm = bench.bench_params(k)
    ids, dist, st = knn.knn_build_ex(Xg, prm)
    # --- properties over all n rows (checked with torch on the outputs)
    assert int(ids.min()) >= 0 and int(ids.max()) < n
    ar = torch.arange(n, device="cuda", dtype=torch.int32)[:, None]
    assert not bool((ids == ar).any()), "self in list"
    srt = torch.sort(ids, dim=1).values
    assert not bool((srt[:, 1:] == srt[:, :-1]).any()), "duplicate id"
    assert bool((dist[:, 1:] >= dist[:, :-1]).all()), "not sorted"
    ties = dist[:, 1:] == dist[:, :-1]
    assert bool((ids[:, 1:][ties] > ids[:, :-1][ties]).all()), "ties not ordered by id"
    # --- sampled rows against the oracle, one by one
    rows = inputs.sample_rows(n, 24, seed=3)
    ids_s = ids[torch.from_numpy(rows).cuda()].cpu().numpy()
    dist_s = dist[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    for q, r in enumerate(rows):
        for j in range(k):
            ref = oracle.distance(X, 0, int(r), int(ids_s[q, j]))
            assert dist_s[q, j] == ref          # byte-valued features: fp32 is exact
    truth, _ = oracle.brute_force_knn(X, k, 0, rows)
    gi, gd = knn.exact_knn(Xg, k, "l2", torch.from_numpy(rows))
    assert (gi.cpu().numpy() == truth).all(), "exact k-NN ids differ from the CPU's"
    # --- recall on a larger sample, ground truth from the (just verified) exhaustive GPU search
    rows2 = inputs.sample_rows(n, 2000, seed=4)
    ti, _ = knn.exact_knn(Xg, k, "l2", torch.from_numpy(rows2))
    rec = oracle.recall(ids[torch.from_numpy(rows2).cuda()].cpu().numpy(), ti.cpu().numpy())
    assert rec >= 0.95, rec
    assert st["rounds_phase1"] == prm.it1 and st["rounds_phase2"] == prm.it2
    # --- the next step on the full-size graph, in the launch configuration the benchmark times: rank-based
    # pruning of all rows; the rows of the first 20 000 nodes (which reach into the whole graph) against the oracle
    pruned, cnt = knn.prune_rank(ids, k // 2, want_counts=True)
    want, want_cnt = oracle.prune_rank(ids.cpu().numpy(), k // 2, n_do=20000)
    assert (pruned[:20000].cpu().numpy() == want).all() and (cnt[:20000].cpu().numpy() == want_cnt).all()
    # properties that hold for every row: kept ids come from the row, none twice; counts bounded by the position
    both = torch.cat([pruned, ids], dim=1).sort(dim=1).values
    assert int((both[:, 1:] == both[:, :-1]).sum()) == n * (k // 2)
    assert bool((cnt <= torch.arange(k, device="cuda")[None, :]).all()) and bool((cnt[:, 0] == 0).all())
    # --- distance-based pruning of the same graph, as the benchmark runs it (Vamana's rule over the neighbours,
    # NSG's over two hops); byte-valued features: the rows of the first nodes must equal the oracle's bit for bit
    ids_h = ids.cpu().numpy()
    for hops, alpha, n_do in ((1, 1.2, 20000), (2, 1.0, 3000)):
        out, deg = knn.prune_dist(Xg, ids, k, alpha=alpha, hops=hops, want_degrees=True)
        want, want_deg, _ = oracle.filter_dist(X, ids_h, hops, 64, alpha, k, n_do=n_do)
        assert (out[:n_do].cpu().numpy() == want).all() and (deg[:n_do].cpu().numpy() == want_deg).all()
        # every row: degree within bounds, the nearest neighbour first, padding only behind the kept ids
        assert int(deg.min()) >= 1 and int(deg.max()) <= k
        if hops == 1:       # (two hops of an approximate graph can reach something nearer than the row's first)
            assert bool((out[:, 0] == ids[:, 0]).all())
        pad = out < 0
        assert bool((pad.sum(dim=1) == k - deg).all()) and bool((pad[:, 1:] >= pad[:, :-1]).all())
        if hops == 1:
            # kept ids come from the row, none twice (padding made distinct so that it pairs with nothing)
            distinct = torch.where(pad, -2 - torch.arange(k, device="cuda", dtype=torch.int32)[None, :], out)
            merged = torch.cat([distinct, ids], dim=1).sort(dim=1).values
            assert int((merged[:, 1:] == merged[:, :-1]).sum()) == int(deg.sum())
