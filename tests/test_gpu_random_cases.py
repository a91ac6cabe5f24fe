"""Many small random cases of the steps that work on finished lists (both prunings and the merge), each
compared with the oracle bit for bit: shapes that no hand-picked case covers (tiny n, k above n, odd d,
cand_size and d_out at their limits, rows full of padding)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import knn

pytestmark = pytest.mark.gpu


def _graph(rng, n, k):
    """Rows of random ids with padding, ids without a node, repeats and self ids mixed in."""
    ids = rng.integers(0, n, size=(n, k)).astype(np.int32)
    noise = rng.random((n, k))
    ids[noise < 0.08] = -1
    ids[(noise >= 0.08) & (noise < 0.11)] = n + rng.integers(0, 5)
    return ids


def test_distance_pruning_random_cases():
    rng = np.random.default_rng(2024)
    for case in range(60):
        n = int(rng.integers(2, 300))
        d = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 31, 33, 64, 100, 128, 129, 200]))
        hops = int(rng.integers(1, 3))
        k = int(rng.integers(1, 65))
        cand_size = int(rng.integers(1, 65))
        d_out = int(rng.integers(1, 65))
        alpha = float(rng.choice([1.0, 1.0, 1.1, 1.5, 3.0]))
        X = rng.integers(0, 40, size=(n, d)).astype(np.float32)           # exact in fp32, many ties and twins
        ids = _graph(rng, n, k)
        want, want_deg, _ = oracle.filter_dist(X, ids, hops, cand_size, alpha, d_out)
        out, deg = knn.prune_dist(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), d_out, alpha=alpha, hops=hops,
                                  cand_size=cand_size, want_degrees=True)
        where = dict(case=case, n=n, d=d, k=k, hops=hops, cand_size=cand_size, d_out=d_out, alpha=alpha)
        assert (out.cpu().numpy() == want).all(), where
        assert (deg.cpu().numpy() == want_deg).all(), where


def test_angle_pruning_random_cases():
    rng = np.random.default_rng(2027)
    for case in range(60):
        n = int(rng.integers(2, 300))
        d = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 31, 33, 64, 100, 128, 129, 200]))
        hops = int(rng.integers(1, 3))
        k = int(rng.integers(1, 65))
        cand_size = int(rng.integers(1, 65))
        d_out = int(rng.integers(1, 65))
        gamma = float(rng.choice([60.0, 60.0, 15.0, 45.0, 72.5, 90.0]))
        X = rng.integers(0, 40, size=(n, d)).astype(np.float32)           # exact in fp32, many right angles and twins
        ids = _graph(rng, n, k)
        want, want_deg, _ = oracle.filter_angle(X, ids, hops, cand_size, gamma, d_out)
        out, deg = knn.prune_angle(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), d_out, gamma_deg=gamma, hops=hops,
                                   cand_size=cand_size, want_degrees=True)
        where = dict(case=case, n=n, d=d, k=k, hops=hops, cand_size=cand_size, d_out=d_out, gamma=gamma)
        assert (out.cpu().numpy() == want).all(), where
        assert (deg.cpu().numpy() == want_deg).all(), where


def test_dispersion_pruning_random_cases():
    rng = np.random.default_rng(2028)
    for case in range(60):
        n = int(rng.integers(2, 300))
        d = int(rng.choice([1, 2, 3, 4, 7, 8, 12, 16, 31, 33, 64, 100, 128, 129, 200]))
        hops = int(rng.integers(1, 3))
        k = int(rng.integers(1, 65))
        cand_size = int(rng.integers(1, 65))
        d_out = int(rng.integers(1, 65))
        X = rng.integers(0, 40, size=(n, d)).astype(np.float32)           # exact in fp32, many equal sums and twins
        ids = _graph(rng, n, k)
        want, want_deg, _ = oracle.filter_dpg(X, ids, hops, cand_size, d_out)
        out, deg = knn.prune_dispersion(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), d_out, hops=hops,
                                        cand_size=cand_size, want_degrees=True)
        where = dict(case=case, n=n, d=d, k=k, hops=hops, cand_size=cand_size, d_out=d_out)
        assert (out.cpu().numpy() == want).all(), where
        assert (deg.cpu().numpy() == want_deg).all(), where


def test_rank_pruning_random_cases():
    rng = np.random.default_rng(2025)
    for case in range(60):
        n = int(rng.integers(1, 400))
        k = int(rng.integers(1, 65))
        d_out = int(rng.integers(1, k + 1))
        ids = _graph(rng, n, k)
        want, want_cnt = oracle.prune_rank(ids, d_out)
        out, cnt = knn.prune_rank(torch.from_numpy(ids).cuda(), d_out, want_counts=True)
        where = dict(case=case, n=n, k=k, d_out=d_out)
        assert (cnt.cpu().numpy() == want_cnt).all(), where
        assert (out.cpu().numpy() == want).all(), where


def test_merge_random_cases():
    rng = np.random.default_rng(2026)
    for case in range(60):
        n = int(rng.integers(1, 300))
        k = int(rng.integers(1, 65))
        kl = int(rng.integers(1, 65))
        w_ids = np.full((n, k), -1, dtype=np.int32)
        w_dist = np.full((n, k), np.inf, dtype=np.float32)
        g_ids, g_dist = knn.lists_clear(n, k)
        for step in range(int(rng.integers(1, 5))):
            nl = int(rng.integers(0, n + 1))
            l2g = rng.permutation(n)[:nl].astype(np.int32)
            l_ids = rng.integers(-1, max(nl, 1) + 2, size=(nl, kl)).astype(np.int32)
            l_dist = rng.integers(0, 30, size=(nl, kl)).astype(np.float32)
            where = dict(case=case, step=step, n=n, k=k, kl=kl, nl=nl)
            if nl:
                oracle.merge_local(w_ids, w_dist, l_ids, l_dist, l2g)
            knn.merge_local(g_ids, g_dist, torch.from_numpy(l_ids).cuda().reshape(nl, kl), torch.from_numpy(l_dist).cuda().reshape(nl, kl),
                            torch.from_numpy(l2g).cuda())
            assert (g_ids.cpu().numpy() == w_ids).all(), where
            assert (g_dist.cpu().numpy() == w_dist).all(), where


def test_whole_build_random_cases():
    """The hot path itself under random shapes and parameters: the finished graph (ids and distances) must equal
    the oracle's on integer-valued data, whatever the dimension, list length, caps, slot count, retention groups
    and round counts."""
    rng = np.random.default_rng(2027)
    for case in range(36):
        n = int(rng.integers(70, 1600))
        d = int(rng.choice([1, 2, 3, 5, 8, 16, 24, 31, 32, 48, 64, 65, 96, 100, 128, 130, 200, 256]))
        k = int(rng.choice([1, 2, 5, 8, 10, 16, 17, 24, 32, 33, 40, 48, 64]))
        k = min(k, n - 1)
        kw = dict(C=int(rng.choice([16, 32, 64, 128, 256])), parts=int(rng.choice([1, 2, 4, 8])),
                  m=int(rng.integers(1, 5)), S=int(rng.integers(1, 33)), R=int(rng.integers(0, 33)))
        it1, it2 = int(rng.integers(0, 4)), int(rng.integers(0, 4))
        shrink = 1 if d <= 128 else 4                                   # squared norms stay below 2^23
        X = np.floor(rng.integers(0, 256, size=(n, d)) / shrink).astype(np.float32)
        metric = str(rng.choice(["l2", "l2", "ip"]))                     # both are exact on these integers
        prm = knn.default_params(k, 6, metric=metric, seed=int(rng.integers(1, 1000)), it1=it1, it2=it2, **kw)
        ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        o = oracle.NNDescent(X, k, metric=knn.METRICS[metric], **oracle.device_model(prm))
        o.run(it1, it2)
        oi, od, _ = o.graph()
        where = dict(case=case, n=n, d=d, k=k, metric=metric, it1=it1, it2=it2, seed=int(prm.seed), **kw)
        assert (ids.cpu().numpy() == oi).all(), where
        assert (dist.cpu().numpy().astype(np.float64) == od).all(), where


@pytest.mark.parametrize("metric", ["l2", "ip"])               # the two metrics whose fp32 arithmetic is exact on integers
def test_whole_build_with_ties_everywhere(metric):
    """A few values in a few dimensions: many points coincide and most distances are shared by many pairs, so nearly
    every threshold is met exactly by candidates with smaller and with larger ids.  The join lets a candidate at the
    threshold's own distance through whatever its id and leaves the rest to the list update; the lists must still be
    the oracle's, entry by entry, after every kind of round."""
    rng = np.random.default_rng(31)
    for n, d, k, vals in ((900, 2, 8, 6), (1500, 3, 20, 4), (700, 5, 33, 3)):
        X = rng.integers(1, 1 + vals, size=(n, d)).astype(np.float32)
        for it1, it2 in ((3, 0), (2, 2)):
            prm = knn.default_params(k, 4, metric=metric, seed=7, it1=it1, it2=it2, C=128)
            ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
            o = oracle.NNDescent(X, k, metric=knn.METRICS[metric], **oracle.device_model(prm))
            o.run(it1, it2)
            oi, od, _ = o.graph()
            where = dict(n=n, d=d, k=k, it1=it1, it2=it2)
            assert (ids.cpu().numpy() == oi).all(), where
            assert (dist.cpu().numpy().astype(np.float64) == od).all(), where


@pytest.mark.parametrize("d,join_f16", [(4096, 0), (4096, 1), (4093, 0), (2050, 2)])
def test_longest_rows(d, join_f16):
    """Rows at the documented maximum length (and just below, unaligned): the whole build against the oracle."""
    rng = np.random.default_rng(d)
    n, k = 300, 8
    X = rng.integers(0, 4, size=(n, d)).astype(np.float32)
    prm = knn.default_params(k, 4, seed=2, C=32, join_f16=join_f16)
    ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = oracle.NNDescent(X, k, **oracle.device_model(prm))
    o.run(prm.it1, prm.it2)
    oi, od, _ = o.graph()
    assert (ids.cpu().numpy() == oi).all()
    assert (dist.cpu().numpy().astype(np.float64) == od).all()
