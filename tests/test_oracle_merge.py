"""Pins of the oracle for merging local indexes into the global one (section 6.1): what the union of
k-NN lists must be is fixed by the definition of "the k nearest"."""
import numpy as np
import pytest

import oracle


def empty(n, k):
    return np.full((n, k), -1, dtype=np.int32), np.full((n, k), np.inf, dtype=np.float32)


def local_index(X, members, k):
    """Exact k-NN lists of the points `members` among themselves, in local numbering."""
    ids, dist = oracle.brute_force_knn(X[members], k)
    return ids, dist.astype(np.float32)


def test_hand_made_example():
    # global node 5 holds (dist, id) = (1, 7), (4, 2), (9, 8); the local index knows node 5 as local 0 with
    # neighbours local 1 (= global 2, dist 4: already there), local 2 (= global 3, dist 2), local 3 (= global 9, dist 9)
    g_ids, g_dist = empty(10, 3)
    g_ids[5] = (7, 2, 8)
    g_dist[5] = (1, 4, 9)
    l2g = np.array([5, 2, 3, 9], dtype=np.int32)
    l_ids = np.array([[1, 2, 3], [0, 2, 3], [0, 1, 3], [0, 1, 2]], dtype=np.int32)
    l_dist = np.array([[4, 2, 9], [4, 1, 1], [2, 1, 1], [9, 1, 1]], dtype=np.float32)
    oracle.merge_local(g_ids, g_dist, l_ids, l_dist, l2g)
    assert list(g_ids[5]) == [7, 3, 2] and list(g_dist[5]) == [1, 2, 4]      # (9, 8) and (9, 9) fall out, 2 counts once
    assert list(g_ids[2]) == [3, 9, 5] and list(g_dist[2]) == [1, 1, 4]      # first touch: the translated local list
    assert (g_ids[[0, 1, 4, 6, 7, 8]] == -1).all()                           # nodes outside the cluster are untouched


def test_overlapping_intervals_of_a_line_give_the_exact_lists():
    # points 0..n-1 on a line, clusters = overlapping intervals.  A node whose k nearest all lie inside one of its
    # clusters gets exactly its global k nearest after the merge, whatever else was merged
    n, k = 200, 6
    X = np.arange(n, dtype=np.float32)[:, None]
    truth, tdist = oracle.brute_force_knn(X, k)
    g_ids, g_dist = empty(n, k)
    clusters = [np.arange(lo, min(n, lo + 60), dtype=np.int32) for lo in range(0, n, 40)]
    for c in clusters:
        l_ids, l_dist = local_index(X, c, k)
        oracle.merge_local(g_ids, g_dist, l_ids, l_dist, c)
    assert (g_ids == truth).all() and (g_dist == tdist.astype(np.float32)).all()


def test_order_of_the_clusters_does_not_matter_and_merging_twice_changes_nothing():
    rng = np.random.default_rng(3)
    n, d, k = 300, 4, 8
    X = rng.integers(0, 30, size=(n, d)).astype(np.float32)
    clusters = [np.sort(rng.permutation(n)[:120]).astype(np.int32) for _ in range(5)]
    locs = [local_index(X, c, k) for c in clusters]
    results = []
    for order in ([0, 1, 2, 3, 4], [4, 2, 0, 3, 1], [1, 1, 3, 0, 4, 2, 2]):
        g_ids, g_dist = empty(n, k)
        for c in order:
            oracle.merge_local(g_ids, g_dist, locs[c][0], locs[c][1], clusters[c])
        results.append((g_ids, g_dist))
    for g_ids, g_dist in results[1:]:
        assert (g_ids == results[0][0]).all() and (g_dist == results[0][1]).all()
    # every row: sorted by (dist, id), no id twice, never the node itself, distances are the true ones
    g_ids, g_dist = results[0]
    for v in range(n):
        row = [(g_dist[v, j], g_ids[v, j]) for j in range(k) if g_ids[v, j] >= 0]
        assert row == sorted(row) and len({i for _, i in row}) == len(row) and v not in {i for _, i in row}
        for dist, i in row:
            assert dist == np.float32(((X[v].astype(np.float64) - X[i]) ** 2).sum())
        assert (g_ids[v, len(row):] == -1).all() and np.isinf(g_dist[v, len(row):]).all()
    # and equals the k nearest among the union of the node's clusters
    for v in range(0, n, 7):
        pool = sorted({int(u) for c in clusters if v in c for u in c if u != v})
        if not pool:
            assert (g_ids[v] == -1).all()
            continue
        dist = ((X[pool].astype(np.float64) - X[v]) ** 2).sum(1).astype(np.float32)
        order = np.lexsort((np.array(pool), dist))[:k]
        assert list(g_ids[v, :len(order)]) == [pool[j] for j in order]


def test_padding_self_and_bad_ids_are_no_entries():
    g_ids, g_dist = empty(6, 4)
    g_ids[0, :2] = (3, 3)                     # an id twice in the global row counts once
    g_dist[0, :2] = (5, 5)
    l2g = np.array([0, 4, 2], dtype=np.int32)
    l_ids = np.array([[1, -1, 7, 0], [0, 2, -1, -1], [0, 1, -1, -1]], dtype=np.int32)
    l_dist = np.array([[2, 0, 0, 0], [2, 3, 0, 0], [6, 3, 0, 0]], dtype=np.float32)
    oracle.merge_local(g_ids, g_dist, l_ids, l_dist, l2g)
    assert list(g_ids[0]) == [4, 3, -1, -1] and list(g_dist[0][:2]) == [2, 5] and np.isinf(g_dist[0][2:]).all()
    with pytest.raises(ValueError):
        oracle.merge_local(g_ids, g_dist, l_ids, l_dist, np.array([0, 9, 2], dtype=np.int32))
