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
    # --- dispersion pruning (DPG's rule: half of the neighbours stay), the same way
    out, deg = knn.prune_dispersion(Xg, ids, k // 2, want_degrees=True)
    want, want_deg, _ = oracle.filter_dpg(X, ids_h, 1, 64, k // 2, n_do=20000)
    assert (out[:20000].cpu().numpy() == want).all() and (deg[:20000].cpu().numpy() == want_deg).all()
    assert bool((deg == k // 2).all()) and bool((out[:, 0] == ids[:, 0]).all())
    merged = torch.cat([out, ids], dim=1).sort(dim=1).values          # kept ids come from the row, none twice
    assert int((merged[:, 1:] == merged[:, :-1]).sum()) == n * (k // 2)
    # --- angle-based pruning (NSSG's rule at 60 degrees over the neighbours), the same way
    out, deg = knn.prune_angle(Xg, ids, k, gamma_deg=60.0, want_degrees=True)
    want, want_deg, _ = oracle.filter_angle(X, ids_h, 1, 64, 60.0, k, n_do=20000)
    assert (out[:20000].cpu().numpy() == want).all() and (deg[:20000].cpu().numpy() == want_deg).all()
    assert int(deg.min()) >= 1 and int(deg.max()) <= k and bool((out[:, 0] == ids[:, 0]).all())
    pad = out < 0
    assert bool((pad.sum(dim=1) == k - deg).all()) and bool((pad[:, 1:] >= pad[:, :-1]).all())


def test_more_nodes_than_one_launch_can_carry():
    # a launch holds fewer than 2^32 work-items, a wave per node reaches that at 2^26 nodes: the kernels that work
    # that way are launched in chunks.  Small rows keep this at a few GB; every row of the result is checked on the
    # device, the last rows (past 2^26) also entry by entry.
    n, d, k = (1 << 26) + 5000, 4, 4
    gen = torch.Generator(device="cuda").manual_seed(5)
    Xg = torch.randint(0, 64, (n, d), generator=gen, device="cuda").to(torch.float32)
    prm = knn.default_params(k, 2, seed=1, it1=1, it2=1, C=16)
    prm.R = 4
    ids, dist, st = knn.knn_build_ex(Xg, prm)
    assert st["rounds_phase1"] == 1 and st["rounds_phase2"] == 1
    assert int(ids.min()) >= 0 and int(ids.max()) < n
    ar = torch.arange(n, device="cuda", dtype=torch.int32)[:, None]
    assert not bool((ids == ar).any())
    srt = torch.sort(ids, dim=1).values
    assert not bool((srt[:, 1:] == srt[:, :-1]).any())
    assert bool((dist[:, 1:] >= dist[:, :-1]).all())
    del srt, ar
    for lo in (0, (1 << 24) - 2000, (1 << 26) - 2000, n - 4000):           # around the chunk borders and at the very end
        rows = slice(lo, lo + 4000)
        ref = ((Xg[rows][:, None, :] - Xg[ids[rows].long()]) ** 2).sum(dim=2)
        assert bool((ref == dist[rows]).all())
    # better than the random start: the mean distance of the lists dropped over the two rounds, everywhere
    assert float(dist[-5000:].mean()) < 0.8 * float(((Xg[-5000:] - Xg[:5000]) ** 2).sum(dim=1).mean())


def test_reverse_samples_over_several_launches_of_the_bucket_step():
    # 1.3 M nodes are 10 157 buckets of 128 targets, more than one launch of the bucket step counts in LDS (8 192):
    # the step runs twice, each launch taking the edges whose targets it covers.  Tiny rows and lists keep the oracle
    # fast; blocks around the border between the two launches and at both ends, then a whole round, bit for bit.
    n, d, k = 1_300_000, 4, 4
    X = np.random.Generator(np.random.PCG64(11)).integers(0, 64, size=(n, d)).astype(np.float32)
    prm = knn.default_params(k, 2, seed=3, C=16)
    prm.R = 4
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    o = oracle.NNDescent(X, k, **oracle.device_model(prm))
    b.init()
    o.init()
    assert (b.graph()[0].cpu().numpy() == o.graph()[0]).all()
    blk, sizes = b.sample_blocks()
    o.phase1_sample()
    border = 8192 * 128
    for lo in (0, border - 1500, n - 3000):
        bl, sz = blk[lo:lo + 3000].cpu().numpy(), sizes[lo:lo + 3000].cpu().numpy()
        for i in range(3000):
            N, O = o.block(lo + i)
            assert sz[i, 0] == len(N) and sz[i, 1] == len(O), lo + i
            assert (bl[i, :len(N)] == N).all() and (bl[i, len(N):len(N) + len(O)] == O).all(), lo + i
    del blk, sizes
    assert b.phase1_round() == o.phase1_round()
    gi, gd, gf = b.graph()
    oi, od, of = o.graph()
    assert (gi.cpu().numpy() == oi).all() and (gd.cpu().numpy().astype(np.float64) == od).all() and (gf.cpu().numpy() == of).all()
    b.close()


def test_c2_full_size_blocks_and_adjacency():
    # The sampler and the adjacency kernel at the benchmark's size and parameters, on lists that two rounds have shaped:
    # the blocks of sampled anchors against the oracle's (which samples the same imported lists), and the adjacency words
    # of those blocks against the lists themselves.
    cfg = inputs.CONFIGS["C2"]
    n, k = cfg["n"], cfg["k"]
    X = inputs.make("C2")
    Xg = torch.from_numpy(X).cuda()
    import bench
    prm = bench.bench_params(k)
    b = knn.Builder(Xg, prm)
    b.init()
    b.phase1_round(False)
    b.phase1_round(False)
    gi, gd, gf = b.graph()
    b.close()
    b = knn.Builder(Xg, prm)                      # a fresh build takes the lists over: both sides sample as in a first round
    b.set_graph(gi, gd, gf)
    ids_h = gi.cpu().numpy()
    o = oracle.NNDescent(X, k, **oracle.device_model(prm))
    o.set_graph(ids_h, gd.cpu().numpy().astype(np.float64), gf.cpu().numpy())
    blk, sizes = b.sample_blocks()
    adj = b.block_adjacency()
    o.phase1_sample()
    rows = np.concatenate([inputs.sample_rows(n, 400, seed=6), np.arange(n - 50, n)])
    rg = torch.from_numpy(rows).cuda()
    bl, sz, ad = blk[rg].cpu().numpy(), sizes[rg].cpu().numpy(), adj[rg].cpu().numpy().view(np.uint32)
    del blk, sizes, adj
    large = 0
    for i, v in enumerate(rows):
        N, O = o.block(int(v))
        nT = len(N) + len(O)
        assert sz[i, 0] == len(N) and sz[i, 1] == len(O), v
        assert (bl[i, :len(N)] == N).all() and (bl[i, len(N):nT] == O).all() and (bl[i, nT:] == -1).all(), v
        if len(N) == 0 or nT < 2:
            assert not ad[i].any()
            continue
        large += nT > 64
        pos = {int(x): p for p, x in enumerate(bl[i, :nT])}
        want = np.zeros((128, 4), dtype=np.uint32)
        for p in range(nT):
            for c in ids_h[bl[i, p]]:
                x = pos.get(int(c))
                if x is not None:
                    want[p, x >> 5] |= np.uint32(1 << (x & 31))
        assert (ad[i] == want).all(), v
    assert large > 0          # (blocks of both kinds of kernel are among the sampled ones)
    b.close()
