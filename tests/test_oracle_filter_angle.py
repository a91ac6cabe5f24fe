"""Pins of the oracle for the angle-based pruning (the NSSG rule of section 3.2 inside the
Collect-Filter-Store procedure of section 5.1): closed forms on a line and on a circle, the strict
inequality at a right angle and at 60 degrees, angles measured here with arccos, the equivalence
with the distance rule on a sphere around p, and invariance under scaling and rotation."""
import math

import numpy as np
import pytest

import oracle
from test_oracle_filter import circle, exact_graph


def test_line_keeps_one_neighbour_per_side():
    # on a line every farther point of a side lies at angle 0 from the nearest one of that side
    n, k = 30, 6
    X = np.arange(n, dtype=np.float32)[:, None]
    for gamma in (1.0, 60.0, 90.0):
        out, deg, _ = oracle.filter_angle(X, exact_graph(X, k), 1, 64, gamma, 4)
        for p in range(n):
            assert list(out[p, :deg[p]]) == [q for q in (p - 1, p + 1) if 0 <= q < n]
            assert (out[p, deg[p]:] == -1).all()


@pytest.mark.parametrize("gamma,want", [
    # nodes 1..9 at 0, 40, .., 320 degrees around p, taken in this order
    (30.0, [1, 2, 3, 4, 5, 6, 7, 8, 9]),      # 40 > 30: nothing is dropped
    (60.0, [1, 3, 5, 7]),                      # 80 apart; node 9 is 40 from node 1
    (85.0, [1, 4, 7]),                         # 120 apart
    (90.0, [1, 4, 7]),
])
def test_circle(gamma, want):
    X, ids = circle(40.0, 9)
    out, deg, _ = oracle.filter_angle(X, ids, 1, 64, gamma, 9, n_do=1)
    assert list(out[0, :deg[0]]) == want


def test_strict_at_a_right_angle():
    # p = (0,0), r = (1,0), c = (0,2): exactly 90 degrees, which does not exceed gamma = 90;
    # c = (-0.25, 2) is past it.  All coordinates and squares are exact in float.
    X = np.array([[0, 0], [1, 0], [0, 2]], dtype=np.float32)
    ids = np.array([[1, 2], [0, 2], [0, 1]], dtype=np.int32)
    out, deg, m = oracle.filter_angle(X, ids, 1, 8, 90.0, 2, n_do=1)
    assert list(out[0]) == [1, -1] and m[0] == 0.0
    X[2] = (-0.25, 2)
    out, deg, _ = oracle.filter_angle(X, ids, 1, 8, 90.0, 2, n_do=1)
    assert list(out[0]) == [1, 2]
    # an obtuse angle passes for every gamma, an angle of zero for none
    out, deg, _ = oracle.filter_angle(X, ids, 1, 8, 5.0, 2, n_do=1)
    assert list(out[0]) == [1, 2]
    X[2] = (3, 0)
    out, deg, _ = oracle.filter_angle(X, ids, 1, 8, 5.0, 2, n_do=1)
    assert list(out[0]) == [1, -1]


def test_threshold_between_two_angles():
    # c at 59 and at 61 degrees from r, gamma = 60
    for ang, kept in ((59.0, False), (61.0, True)):
        a = math.radians(ang)
        X = np.array([[0, 0], [1, 0], [1.5 * math.cos(a), 1.5 * math.sin(a)]], dtype=np.float32)
        ids = np.array([[1, 2], [0, 2], [0, 1]], dtype=np.int32)
        out, deg, _ = oracle.filter_angle(X, ids, 1, 8, 60.0, 2, n_do=1)
        assert (deg[0] == 2) == kept


@pytest.mark.parametrize("hops,gamma", [(1, 60.0), (1, 35.0), (2, 60.0), (2, 75.0)])
def test_angles_measured_with_arccos(hops, gamma):
    rng = np.random.default_rng(11)
    n, d, k, d_out, cs = 400, 6, 12, 8, 40
    X = (rng.normal(size=(n, d)) * 3).astype(np.float32)
    ids = exact_graph(X, k)
    out, deg, margin = oracle.filter_angle(X, ids, hops, cs, gamma, d_out)
    Xd = X.astype(np.float64)
    eps = 1e-4                              # degrees; decisions nearer the threshold are not judged

    def angle(p, a, b):
        u, v = Xd[a] - Xd[p], Xd[b] - Xd[p]
        c = u @ v / math.sqrt((u @ u) * (v @ v))
        return math.degrees(math.acos(max(-1.0, min(1.0, c))))

    def key(p, c):
        return (np.float32(((Xd[p] - Xd[c]) ** 2).sum()), c)

    seen_drop = 0
    for p in range(n):
        R = [int(c) for c in out[p, :deg[p]]]
        assert len(set(R)) == len(R) and p not in R and (out[p, deg[p]:] == -1).all()
        assert all(key(p, R[i]) < key(p, R[i + 1]) for i in range(len(R) - 1))
        for j in range(len(R)):
            for i in range(j):
                assert angle(p, R[i], R[j]) > gamma - eps
        cand = set(ids[p].tolist())
        if hops == 2:
            for u in ids[p]:
                cand |= set(ids[u].tolist())
        cand.discard(p)
        cand = sorted(cand, key=lambda c: key(p, c))[:cs]
        horizon = len(cand) if deg[p] < d_out else cand.index(R[-1])
        for c in cand[:horizon]:
            if c in R:
                continue
            seen_drop += 1
            before = [r for r in R if key(p, r) < key(p, c)]
            assert any(angle(p, r, c) <= gamma + eps for r in before)
    assert seen_drop > n                    # the rule did drop candidates
    out_s, _, _ = oracle.filter_angle(X, ids, hops, cs, gamma, 3)
    assert (out_s == out[:, :3]).all()
    out_2, _, _ = oracle.filter_angle(X * 2, ids, hops, cs, gamma, d_out)      # a power of two: same roundings
    assert (out_2 == out).all()


def test_same_as_distance_rule_on_a_sphere():
    # candidates at one distance from p: |p c| < alpha |r c|  <=>  angle(r, c) > 2 asin(1 / (2 alpha))
    rng = np.random.default_rng(12)
    m, d = 40, 5
    for alpha in (1.0, 1.2, 1.6):
        gamma = math.degrees(2 * math.asin(1 / (2 * alpha)))
        for trial in range(60):
            V = rng.normal(size=(m, d))
            V /= np.linalg.norm(V, axis=1, keepdims=True)
            X = np.vstack([np.zeros((1, d)), V]).astype(np.float32)
            ids = np.tile(np.arange(1, m + 1, dtype=np.int32), (m + 1, 1))
            # the order among the candidates is decided by roundings of 1.0, but both rules see the same
            # order; a pair within rounding of the threshold would show as a difference (none with this seed)
            a, dega, _ = oracle.filter_dist(X, ids, 1, 64, alpha, m, n_do=1)
            b, degb, _ = oracle.filter_angle(X, ids, 1, 64, gamma, m, n_do=1)
            assert (a == b).all() and dega[0] == degb[0] and 1 < dega[0] < m


def test_rotation_and_translation_leave_robust_rows_alone():
    rng = np.random.default_rng(13)
    n, d, k = 300, 4, 10
    X = rng.normal(size=(n, d)).astype(np.float32)
    ids = exact_graph(X, k)
    out, deg, m = oracle.filter_angle(X, ids, 1, 64, 60.0, k)
    Q, _ = np.linalg.qr(rng.normal(size=(d, d)))
    Y = (X.astype(np.float64) @ Q + 0.5).astype(np.float32)
    out2, deg2, m2 = oracle.filter_angle(Y, ids, 1, 64, 60.0, k)
    robust = (m > 1e-5) & (m2 > 1e-5)
    assert robust.sum() > n // 2
    assert (out[robust] == out2[robust]).all()


def test_bad_arguments():
    X = np.zeros((4, 2), dtype=np.float32)
    ids = np.zeros((4, 2), dtype=np.int32)
    for gamma in (0.0, -1.0, 90.5, float("nan")):
        with pytest.raises(ValueError):
            oracle.filter_angle(X, ids, 1, 8, gamma, 2)
