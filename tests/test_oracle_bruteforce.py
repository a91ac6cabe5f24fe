"""Pins for O-BF, the exhaustive k-NN that is the ground truth of the recall definition
(section 7.1, Metrics) and of every other oracle check."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_mix64_published_vectors():
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64_vectors.txt")) if not l.startswith("#")]
    g = 0x9E3779B97F4A7C15
    got = [oracle.mix64(((i + 1) * g) & (2**64 - 1)) for i in range(len(want))]
    assert got == want


def test_hash3_is_three_nested_mixes():
    M = 2**64 - 1
    g = 0x9E3779B97F4A7C15
    for seed, tag, x, y in [(0, 1, 0, 0), (123456789, 7, 42, 99), (M, 3, 2**31 - 1, 5)]:
        h = oracle.mix64((seed + tag * g) & M)
        h = oracle.mix64((h + x) & M)
        h = oracle.mix64((h + y) & M)
        assert oracle.hash3(seed, tag, x, y) == h


def test_line_closed_form():
    # points 0..n-1 on a line: neighbours of i are i-1, i+1, i-2, i+2, ... (smaller id first on ties)
    n, k = 50, 6
    X = np.arange(n, dtype=np.float32).reshape(n, 1)
    ids, dist = oracle.brute_force_knn(X, k)
    for i in range(n):
        cand = sorted((float((i - j) ** 2), j) for j in range(n) if j != i)[:k]
        assert [c[1] for c in cand] == ids[i].tolist()
        assert [c[0] for c in cand] == dist[i].tolist()
    # an interior point explicitly
    assert ids[10].tolist() == [9, 11, 8, 12, 7, 13]
    assert dist[10].tolist() == [1, 1, 4, 4, 9, 9]


def test_grid_closed_form():
    # interior point of a unit grid: squared distances 1 x4, 2 x4, 4 x4, 5 x8
    g = 9
    X = np.array([(x, y) for x in range(g) for y in range(g)], dtype=np.float32)
    ids, dist = oracle.brute_force_knn(X, 20)
    c = 4 * g + 4
    assert dist[c].tolist() == [1] * 4 + [2] * 4 + [4] * 4 + [5] * 8
    # equal distances are ordered by id
    assert ids[c][:4].tolist() == sorted(ids[c][:4].tolist())


@pytest.mark.parametrize("metric", [0, 1, 2])
def test_against_independent_full_sort(metric):
    rng = np.random.default_rng(5 + metric)
    n, d, k = 257, 19, 11
    X = rng.standard_normal((n, d)).astype(np.float32)
    Xd = X.astype(np.float64)
    ids, dist = oracle.brute_force_knn(X, k, metric)
    for i in range(0, n, 7):
        if metric == 0:
            dd = ((Xd - Xd[i]) ** 2).sum(axis=1)
        elif metric == 1:
            dd = -(Xd @ Xd[i])
        else:
            dd = 1.0 - (Xd @ Xd[i]) / np.sqrt((Xd * Xd).sum(axis=1) * (Xd[i] @ Xd[i]))
        dd[i] = np.inf
        order = np.lexsort((np.arange(n), dd))[:k]
        assert order.tolist() == ids[i].tolist()
        np.testing.assert_allclose(dist[i], dd[order], rtol=1e-12, atol=1e-12)


def test_rows_argument_and_symmetry():
    rng = np.random.default_rng(9)
    X = rng.standard_normal((120, 8)).astype(np.float32)
    full_ids, full_d = oracle.brute_force_knn(X, 5)
    rows = np.array([3, 77, 119, 0])
    ids, d = oracle.brute_force_knn(X, 5, rows=rows)
    assert (ids == full_ids[rows]).all() and (d == full_d[rows]).all()
    # the distance function is symmetric and zero on identical rows
    for m in (0, 1, 2):
        assert oracle.distance(X, m, 4, 9) == oracle.distance(X, m, 9, 4)
    assert oracle.distance(X, 0, 4, 4) == 0.0
    assert abs(oracle.distance(X, 2, 4, 4)) < 1e-15


def test_metrics_agree_on_unit_vectors():
    # on unit-norm rows squared L2 = 2 - 2<x,y>: the three metrics rank identically
    rng = np.random.default_rng(11)
    X = rng.standard_normal((200, 12))
    X = (X / np.linalg.norm(X, axis=1, keepdims=True)).astype(np.float32)
    a, _ = oracle.brute_force_knn(X, 8, 0)
    b, _ = oracle.brute_force_knn(X, 8, 1)
    c, _ = oracle.brute_force_knn(X, 8, 2)
    # fp32 rows are unit only to 1e-7, so allow a handful of near-tie swaps
    assert (a != b).mean() < 0.01 and (b != c).mean() < 0.01


def test_recall_definition():
    ids = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.int32)
    truth = np.array([[3, 9, 1], [7, 8, 9]], dtype=np.int32)
    assert oracle.recall(ids, truth) == pytest.approx(2 / 6)
    assert oracle.recall(truth, truth) == 1.0


def test_invalid_k():
    X = np.zeros((5, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.brute_force_knn(X, 5)
