"""Pins of the oracle for the distance-based pruning (NSG / Vamana rule of section 3.2 inside
the Collect-Filter-Store procedure of section 5.1) against what geometry fixes: closed forms on
a line and on a circle, the strict inequality, the limit of a large alpha, duplicates, the 2-hop
candidate set against a set union written here, and invariants of the serial rule."""
import math

import numpy as np
import pytest

import oracle


def exact_graph(X, k):
    ids, _ = oracle.brute_force_knn(X, k)
    return ids


def test_line_nsg_keeps_one_neighbour_per_side():
    # points 0..n-1 on a line: any farther point on the same side is closer to the nearer one
    # than to p, so alpha = 1 keeps exactly p-1 and p+1 (p-1 first: equal distance, smaller id)
    n, k = 40, 8
    X = np.arange(n, dtype=np.float32)[:, None]
    out, deg, _ = oracle.filter_dist(X, exact_graph(X, k), 1, 64, 1.0, 6)
    for p in range(n):
        want = [q for q in (p - 1, p + 1) if 0 <= q < n]
        assert list(out[p, :deg[p]]) == want
        assert (out[p, deg[p]:] == -1).all()


def test_line_two_hops():
    # k = 2 on a line: N(p) = {p-1, p+1}; two hops add p-2 and p+2.  A very large alpha keeps
    # all four in order of distance; alpha = 1 keeps the two nearest only.
    n = 30
    X = np.arange(n, dtype=np.float32)[:, None]
    ids = exact_graph(X, 2)
    out, deg, _ = oracle.filter_dist(X, ids, 2, 64, 1e3, 4)
    for p in range(3, n - 3):
        assert list(out[p]) == [p - 1, p + 1, p - 2, p + 2]
    out, deg, _ = oracle.filter_dist(X, ids, 2, 64, 1.0, 4)
    for p in range(3, n - 3):
        assert list(out[p, :deg[p]]) == [p - 1, p + 1]
    # cand_size cuts the ordered candidates before the filter
    out, deg, _ = oracle.filter_dist(X, ids, 2, 3, 1e3, 4)
    for p in range(3, n - 3):
        assert list(out[p]) == [p - 1, p + 1, p - 2, -1]


def circle(step_deg, m):
    """p = node 0 at the centre, nodes 1..m on a circle at multiples of step_deg, radii growing by
    0.1 % per node so that the order by distance is the order by id."""
    pts = [(0.0, 0.0)]
    for i in range(m):
        r = 1.0 + 0.001 * i
        a = math.radians(step_deg * i)
        pts.append((r * math.cos(a), r * math.sin(a)))
    X = np.array(pts, dtype=np.float32)
    ids = np.tile(np.arange(1, m + 1, dtype=np.int32), (m + 1, 1))
    return X, ids


@pytest.mark.parametrize("alpha,want", [
    # |p c| < alpha |r c| on the unit circle <=> angle(r, c) > 2 asin(1 / (2 alpha)): 60 degrees for
    # alpha = 1, 49.2 for 1.2, 38.9 for 1.5.  Nodes 40 degrees apart: the greedy rule keeps every
    # second one (the last, at 320, is 40 from the first), and all of them once alpha = 1.5.
    (1.0, [1, 3, 5, 7]),
    (1.2, [1, 3, 5, 7]),
    (1.5, [1, 2, 3, 4, 5, 6, 7, 8, 9]),
])
def test_circle_angle_threshold(alpha, want):
    X, ids = circle(40.0, 9)
    out, deg, _ = oracle.filter_dist(X, ids, 1, 64, alpha, 9, n_do=1)
    assert list(out[0, :deg[0]]) == want


def test_strict_inequality():
    # p = (0,0), r = (2,0), c = (1,3): sq(p,c) = sq(r,c) = 10.  The table's rule is a strict "<",
    # so c is not inserted once r is in; with c moved a little away from r it is.
    X = np.array([[0, 0], [2, 0], [1, 3]], dtype=np.float32)
    ids = np.array([[1, 2], [0, 2], [0, 1]], dtype=np.int32)
    out, deg, _ = oracle.filter_dist(X, ids, 1, 8, 1.0, 2, n_do=1)
    assert list(out[0]) == [1, -1]
    X[2] = (0, 3)        # sq(p,c) = 9 < sq(r,c) = 13
    out, deg, _ = oracle.filter_dist(X, ids, 1, 8, 1.0, 2, n_do=1)
    assert list(out[0]) == [1, 2]


def test_large_alpha_is_nearest_candidates():
    # alpha -> infinity: nothing is occluded (no duplicate points here), so the result is the
    # d_out nearest candidates in (distance, id) order
    rng = np.random.default_rng(5)
    n, d, k = 300, 6, 10
    X = rng.integers(0, 50, size=(n, d)).astype(np.float32)
    X += np.arange(n, dtype=np.float32)[:, None] * 1e-3      # no two points equal
    ids = exact_graph(X, k)
    out, deg, _ = oracle.filter_dist(X, ids, 1, 64, 1e6, 7)
    assert (out == ids[:, :7]).all()
    # two hops: union of the rows written out here, ordered by numpy
    out2, deg2, _ = oracle.filter_dist(X, ids, 2, 1000, 1e6, 12)
    for p in range(n):
        s = set(ids[p].tolist())
        for u in ids[p]:
            s |= set(ids[u].tolist())
        s.discard(p)
        c = np.array(sorted(s))
        dist = ((X[c].astype(np.float64) - X[p].astype(np.float64)) ** 2).sum(1).astype(np.float32)
        order = np.lexsort((c, dist))
        assert list(out2[p]) == list(c[order][:12])


def test_two_hops_of_exact_graph_cut_to_k_is_one_hop():
    # on the exact k-NN graph the k nearest of the 2-hop candidates are the neighbours themselves
    rng = np.random.default_rng(6)
    n, d, k = 400, 5, 8
    X = rng.normal(size=(n, d)).astype(np.float32)
    ids = exact_graph(X, k)
    a, dega, _ = oracle.filter_dist(X, ids, 1, k, 1.2, k)
    b, degb, _ = oracle.filter_dist(X, ids, 2, k, 1.2, k)
    assert (a == b).all() and (dega == degb).all()


def test_duplicate_of_a_kept_neighbour_is_never_kept():
    rng = np.random.default_rng(7)
    n, d, k = 60, 4, 12
    X = rng.integers(0, 20, size=(n, d)).astype(np.float32)
    X[1::2] = X[0::2]                     # every point has a twin
    ids = exact_graph(X, k)
    for alpha in (1.0, 1.5, 100.0):
        out, deg, _ = oracle.filter_dist(X, ids, 1, 64, alpha, k)
        for p in range(n):
            kept = [tuple(X[c]) for c in out[p, :deg[p]]]
            assert len(kept) == len(set(kept))


@pytest.mark.parametrize("hops,alpha", [(1, 1.0), (1, 1.3), (2, 1.0), (2, 1.15)])
def test_invariants_of_the_serial_rule(hops, alpha):
    rng = np.random.default_rng(8)
    n, d, k, d_out, cs = 500, 8, 12, 8, 40
    X = (rng.normal(size=(n, d)) * 4).astype(np.float32)
    ids = exact_graph(X, k)
    out, deg, _ = oracle.filter_dist(X, ids, hops, cs, alpha, d_out)
    Xd = X.astype(np.float64)
    a2 = np.float32(alpha) * np.float32(alpha)

    def sq(a, b):
        return np.float32(((Xd[a] - Xd[b]) ** 2).sum())

    for p in range(n):
        R = [int(c) for c in out[p, :deg[p]]]
        assert (out[p, deg[p]:] == -1).all() and deg[p] <= d_out
        assert len(set(R)) == len(R) and p not in R
        dpc = [sq(p, c) for c in R]
        assert all((dpc[i], R[i]) < (dpc[i + 1], R[i + 1]) for i in range(len(R) - 1))   # closest first
        for j in range(len(R)):                   # no kept node occludes a later kept one
            for i in range(j):
                assert dpc[j] < a2 * sq(R[i], R[j])
        # a candidate in front of the last kept node that is missing has an occluder kept before it
        cand = set(ids[p].tolist())
        if hops == 2:
            for u in ids[p]:
                cand |= set(ids[u].tolist())
        cand.discard(p)
        cand = sorted(cand, key=lambda c: (sq(p, c), c))[:cs]
        if deg[p] < d_out:
            horizon = len(cand)
        else:
            horizon = cand.index(R[-1])
        for c in cand[:horizon]:
            if c in R:
                continue
            before = [r for r in R if (sq(p, r), r) < (sq(p, c), c)]
            assert any(not (sq(p, c) < a2 * sq(r, c)) for r in before)
    # a smaller d_out is a prefix; doubling the data changes nothing
    out_s, deg_s, _ = oracle.filter_dist(X, ids, hops, cs, alpha, 3)
    assert (out_s == out[:, :3]).all()
    out_2, _, _ = oracle.filter_dist(X * 2, ids, hops, cs, alpha, d_out)
    assert (out_2 == out).all()


def test_margin_marks_fragile_rows():
    # the isosceles triangle decides on an exact tie: margin 0; moved away, the margin is the gap
    X = np.array([[0, 0], [2, 0], [1, 3]], dtype=np.float32)
    ids = np.array([[1, 2], [0, 2], [0, 1]], dtype=np.int32)
    _, _, m = oracle.filter_dist(X, ids, 1, 8, 1.0, 2, n_do=1)
    assert m[0] == 0.0
    X[2] = (0, 3)
    _, _, m = oracle.filter_dist(X, ids, 1, 8, 1.0, 2, n_do=1)
    # decisions: order (4 vs 9), c against r (9 < 13); norms 0 + 4 + 9
    assert m[0] == pytest.approx(min(5.0, 4.0) / 13.0)


def test_bad_arguments():
    X = np.zeros((4, 2), dtype=np.float32)
    ids = np.zeros((4, 2), dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.filter_dist(X, ids, 3, 8, 1.0, 2)
    with pytest.raises(ValueError):
        oracle.filter_dist(X, ids, 1, 8, 0.5, 2)
