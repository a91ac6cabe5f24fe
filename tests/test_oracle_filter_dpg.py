"""Pins of the oracle for the dispersion pruning (the DPG rule of section 3.2, which section 5.1 reaches
with the angle metric and a threshold of 0): its arc cosine against numpy's, a hand-made example in
the plane, a greedy written here in float64 with numpy's arccos on random data (rows whose decisions
were not close), special cases and invariants."""
import math

import numpy as np
import pytest

import oracle
from test_oracle_filter import exact_graph


def test_angle_against_arccos():
    rng = np.random.default_rng(21)
    P = rng.normal(size=(4000, 3, 5))                       # triangles p, r, c in 5 dimensions
    u, v = P[:, 1] - P[:, 0], P[:, 2] - P[:, 0]
    a, b, c = (u * u).sum(1), (v * v).sum(1), ((P[:, 1] - P[:, 2]) ** 2).sum(1)
    want = np.arccos(np.clip((u * v).sum(1) / np.sqrt(a * b), -1, 1))
    got = oracle.angle_at(a, b, c)
    # the polynomial is good to 2e-8; float rounding of the cosine costs more near 0 and pi
    ok = (want > 0.05) & (want < math.pi - 0.05)
    assert np.abs(got - want)[ok].max() < 3e-6
    assert np.abs(got - want).max() < 1e-3
    # the whole range on unit vectors: c = 2 - 2 cos
    x = np.linspace(-1, 1, 4001)
    got = oracle.angle_at(np.ones_like(x), np.ones_like(x), 2 - 2 * x)
    assert np.abs(got - np.arccos(x)).max() < 2e-6


def test_angle_special_cases():
    f = oracle.angle_at
    assert f([4.0], [9.0], [1.0])[0] == 0.0                 # r and c on one ray: 2, 3, |r c| = 1
    assert f([4.0], [9.0], [25.0])[0] == np.float32(math.pi)   # opposite rays
    assert abs(f([4.0], [9.0], [13.0])[0] - math.pi / 2) < 2e-7    # right angle
    assert f([0.0], [9.0], [9.0])[0] == 0.0                 # r at p's position: no direction
    assert f([4.0], [0.0], [4.0])[0] == 0.0
    assert f([3.0], [5.0], [2.0])[0] == f([5.0], [3.0], [2.0])[0]      # symmetric in r and c
    # the law of cosines with the sign of c: 60 degrees in an equilateral triangle
    assert abs(f([1.0], [1.0], [1.0])[0] - math.pi / 3) < 2e-7
    assert abs(f([1.0], [1.0], [3.0])[0] - 2 * math.pi / 3) < 2e-7


def test_hand_made_example_in_the_plane():
    # p at the origin; A nearest on the x axis, B at 90 degrees, C at 175 degrees, D 9 degrees below the axis.
    # A first; C has the largest angle to A; then D (8.7 + 176.1 = 184.8 degrees) leads B (90 + 85.2 = 175.2).
    X = np.array([[0, 0], [1, 0], [0, 1.1], [-1.2, 0.1], [1.3, -0.2]], dtype=np.float32)
    ids = np.tile(np.array([1, 2, 3, 4], dtype=np.int32), (5, 1))
    out, deg, margin = oracle.filter_dpg(X, ids, 1, 64, 4, n_do=1)
    assert list(out[0]) == [1, 3, 4, 2] and deg[0] == 4
    # the margin is the smaller of that lead (radians) and the relative gaps between the candidates' distances:
    # here the gap between C and D, (1.73 - 1.45) / (1.45 + 1.73)
    assert margin[0] == pytest.approx(min(math.radians(184.8 - 175.2), 0.28 / 3.18), abs=2e-3)
    Y = X * np.array([[1], [1], [2], [4], [8]], dtype=np.float32)      # the same directions, wide gaps between the distances
    out, _, margin = oracle.filter_dpg(Y, ids, 1, 64, 4, n_do=1)
    assert list(out[0]) == [1, 3, 4, 2]
    assert margin[0] == pytest.approx(math.radians(184.8 - 175.2), abs=2e-3)
    out, deg, _ = oracle.filter_dpg(X, ids, 1, 64, 2, n_do=1)
    assert list(out[0]) == [1, 3] and deg[0] == 2
    out, deg, _ = oracle.filter_dpg(X, ids, 1, 3, 4, n_do=1)          # the three nearest only: D is cut
    assert list(out[0]) == [1, 3, 2, -1] and deg[0] == 3


def greedy64(X, cand, p, d_out):
    """The greedy in float64 with numpy's arccos; returns the order and the smallest lead (radians)."""
    Xd = X.astype(np.float64)

    def ang(r, c):
        u, v = Xd[r] - Xd[p], Xd[c] - Xd[p]
        nu, nv = u @ u, v @ v
        if nu == 0 or nv == 0:
            return 0.0
        return math.acos(max(-1.0, min(1.0, u @ v / math.sqrt(nu * nv))))

    R, left, score, lead = [cand[0]], list(cand[1:]), {c: 0.0 for c in cand[1:]}, math.inf
    while left and len(R) < d_out:
        for c in left:
            score[c] += ang(R[-1], c)
        ranked = sorted(left, key=lambda c: -score[c])            # stable: the nearer of equals first
        if len(ranked) > 1:
            lead = min(lead, score[ranked[0]] - score[ranked[1]])
        R.append(ranked[0])
        left.remove(ranked[0])
    return R, lead


@pytest.mark.parametrize("hops,d,d_out,cs", [(1, 3, 6, 64), (1, 8, 12, 64), (2, 5, 10, 30), (1, 16, 5, 9)])
def test_against_a_float64_greedy(hops, d, d_out, cs):
    rng = np.random.default_rng(22)
    n, k = 300, 12
    X = rng.normal(size=(n, d)).astype(np.float32)
    ids = exact_graph(X, k)
    out, deg, margin = oracle.filter_dpg(X, ids, hops, cs, d_out)
    Xd = X.astype(np.float64)
    judged = 0
    for p in range(n):
        cand = set(ids[p].tolist())
        if hops == 2:
            for u in ids[p]:
                cand |= set(ids[u].tolist())
        cand.discard(p)
        cand = sorted(cand, key=lambda c: (np.float32(((Xd[p] - Xd[c]) ** 2).sum()), c))[:cs]
        R, lead = greedy64(X, cand, p, d_out)
        assert deg[p] == min(d_out, len(cand)) and out[p, 0] == cand[0]
        assert sorted(out[p, :deg[p]].tolist()) == sorted(set(out[p, :deg[p]].tolist()))     # no node twice
        assert set(out[p, :deg[p]].tolist()) <= set(cand) and (out[p, deg[p]:] == -1).all()
        if lead > 1e-4:
            judged += 1
            assert list(out[p, :deg[p]]) == R
            assert 0 < margin[p] <= lead + 2e-5                      # the lead, or a smaller gap in the ordering
    assert judged > 0.8 * n
    out_s, _, _ = oracle.filter_dpg(X, ids, hops, cs, 3)                  # greedy: a smaller d_out is a prefix
    assert (out_s == out[:, :3]).all()
    out_2, _, _ = oracle.filter_dpg(X * 4, ids, hops, cs, d_out)          # a power of two: same roundings
    assert (out_2 == out).all()


def test_everything_is_kept_when_there_is_room():
    rng = np.random.default_rng(23)
    n, d, k = 100, 4, 8
    X = rng.normal(size=(n, d)).astype(np.float32)
    ids = exact_graph(X, k)
    out, deg, _ = oracle.filter_dpg(X, ids, 1, 64, k)
    assert (deg == k).all()
    assert (np.sort(out, axis=1) == np.sort(ids, axis=1)).all() and (out[:, 0] == ids[:, 0]).all()


def test_twins_and_a_candidate_at_p():
    # candidate 2 sits on candidate 1, candidate 3 on p itself: both add no angle and come last, the nearer first
    X = np.array([[0, 0, 0], [1, 0, 0], [1, 0, 0], [0, 0, 0], [0, 2, 0], [0, 0, -3]], dtype=np.float32)
    ids = np.tile(np.array([1, 2, 3, 4, 5], dtype=np.int32), (6, 1))
    out, deg, _ = oracle.filter_dpg(X, ids, 1, 64, 5, n_do=1)
    # order by distance: 3 (at p), 1, 2, 4, 5.  3 first (nearest); every angle to it is 0, so 1 follows (nearest of
    # equals); then 4 and 5 at 90 degrees from 1 (4 nearer), then 2, whose angles are 0 + 0 + 90 + 90 against
    # nothing else left
    assert list(out[0]) == [3, 1, 4, 5, 2]


def test_bad_arguments():
    X = np.zeros((4, 2), dtype=np.float32)
    ids = np.zeros((4, 2), dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.filter_dpg(X, ids, 3, 8, 2)
    with pytest.raises(ValueError):
        oracle.filter_dpg(X, ids, 1, 0, 2)
