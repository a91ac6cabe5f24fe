"""Pins of the rank-based pruning oracle (sections 3.2 and 5.2) against things other than itself."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "detour_example.txt")


def _paths_definition(ids):
    """Independent route enumeration: for every directed 2-hop route A -> D and F -> D with D in both rows,
    the route A -> D -> F is a detour of (A, F) when max(pos_A(D), pos_F(D)) < pos_A(F)."""
    n, k = ids.shape
    pos = [{int(u): p + 1 for p, u in enumerate(row)} for row in ids]
    cnt = np.zeros((n, k), dtype=np.int32)
    for a in range(n):
        for f, pf in pos[a].items():
            if not (0 <= f < n):
                continue
            shared = set(pos[a]) & set(pos[f])
            cnt[a, pf - 1] = sum(1 for d in shared if max(pos[a][d], pos[f][d]) < pf)
    return cnt


def test_worked_example_of_the_paper():
    rows, want = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":")
        if key == "A_counts":
            want = [int(x) for x in val.split()]
        else:
            rows[int(key)] = [int(x) for x in val.split()]
    n, k = 11, 5
    ids = np.zeros((n, k), dtype=np.int32)
    for v in range(n):                       # rows the text says nothing about: fillers that share nothing with A
        ids[v] = rows.get(v, [(v + 1 + t) % 5 + 6 if (v + 1 + t) % 5 + 6 != v else 6 for t in range(k)])
    out, cnt = oracle.prune_rank(ids, 4)
    assert cnt[0].tolist() == want
    # F, the only edge with a detour, is the one that goes when A keeps four of its five neighbours
    assert out[0].tolist() == [1, 2, 3, 4]


def test_closed_form_on_cliques():
    """Disjoint cliques of k + 1 nodes, rows in ascending id order: with a, f, d the indices inside the clique,
    pos_X(Y) = y + 1 - [y > x], and D is a detour of (A, F) iff both its positions are below pos_A(F)."""
    k, cliques = 7, 5
    n = cliques * (k + 1)
    ids = np.zeros((n, k), dtype=np.int32)
    for v in range(n):
        base = v - v % (k + 1)
        ids[v] = [base + y for y in range(k + 1) if base + y != v]
    _, cnt = oracle.prune_rank(ids, k)
    for v in range(n):
        a = v % (k + 1)
        for p, fid in enumerate(ids[v]):
            f = fid % (k + 1)
            pos_af = f + 1 - (f > a)
            assert pos_af == p + 1
            want = sum(1 for d in range(k + 1) if d not in (a, f)
                       and d + 1 - (d > a) < pos_af and d + 1 - (d > f) < pos_af)
            assert cnt[v, p] == want, (v, p)


@pytest.mark.parametrize("n,k,seed", [(60, 6, 1), (200, 16, 2), (90, 33, 3)])
def test_equals_the_route_enumeration_on_geometric_graphs(n, k, seed):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, 4)).astype(np.float32)
    ids, _ = oracle.brute_force_knn(X, k)
    _, cnt = oracle.prune_rank(ids, k)
    assert (cnt == _paths_definition(ids)).all()
    assert cnt.sum() > 0                                    # near neighbours do share neighbours
    assert (cnt[:, 0] == 0).all()                           # nothing is closer than the first neighbour
    assert (cnt <= np.arange(k)[None, :]).all()             # at most one detour per closer neighbour


def test_selection_order_ties_and_invalid_ids():
    ids = np.array([[1, 2, 3, 4], [0, 2, 3, 4], [0, 1, 3, 4], [0, 1, 2, 4], [0, 1, 2, 3]], dtype=np.int32)
    out, cnt = oracle.prune_rank(ids, 2)
    order = [sorted(range(4), key=lambda p: (cnt[v, p], p))[:2] for v in range(5)]
    assert out.tolist() == [[int(ids[v, p]) for p in order[v]] for v in range(5)]
    # d_out = k only reorders; rows stay permutations of the input rows
    full, _ = oracle.prune_rank(ids, 4)
    assert all(sorted(full[v]) == sorted(ids[v]) for v in range(5))
    # an id without a row (padding) brings no detours and is kept or dropped by its position alone
    ids2 = ids.copy(); ids2[0, 3] = -1
    _, cnt2 = oracle.prune_rank(ids2, 4)
    assert cnt2[0, 3] == 0
    with pytest.raises(ValueError):
        oracle.prune_rank(ids, 5)


def test_hand_made_rows_reordering_repeats_self_and_ids_without_a_row():
    """Counts and the kept order worked out by hand from the definition (a detour of (A, F), F at position p,
    is a node in front of p in A's row and in front of p in F's row)."""
    n, k = 12, 4
    filler = [8, 9, 10, 11]
    ids = np.array([filler] * n, dtype=np.int32)
    # A = 0: node 3 (position 2) has both closer neighbours in front of its own row: two detours; node 4 none
    ids[0] = [1, 2, 3, 4]
    ids[3] = [1, 2, 8, 9]
    out, cnt = oracle.prune_rank(ids, 3)
    assert cnt[0].tolist() == [0, 0, 2, 0]
    assert out[0].tolist() == [1, 2, 4]                      # the farther node with fewer detours goes first
    full, _ = oracle.prune_rank(ids, 4)
    assert full[0].tolist() == [1, 2, 4, 3]
    # a neighbour shared only at or behind F's position is no detour: node 4 lists 3 too late, node 2 lists 1 in time
    ids[4] = [8, 9, 10, 3]
    ids[2] = [1, 8, 9, 10]
    _, cnt = oracle.prune_rank(ids, 4)
    assert cnt[0].tolist() == [0, 1, 2, 0]
    # F's row names F itself: F is not in front of its own position in A's row
    ids[4] = [4, 8, 9, 10]
    _, cnt = oracle.prune_rank(ids, 4)
    assert cnt[0, 3] == 0
    # A lists a node twice: one detour, not two
    ids[5] = [1, 1, 6, 7]
    ids[6] = [1, 8, 9, 10]
    _, cnt = oracle.prune_rank(ids, 4)
    assert cnt[5].tolist() == [0, 0, 1, 0]
    # the same id without a row (n + 7) in A's row and in F's row is no node, hence no detour
    ids[7] = [1, n + 7, 6, 2]
    ids[6] = [n + 7, 8, 9, 10]
    _, cnt = oracle.prune_rank(ids, 4)
    assert cnt[7].tolist() == [0, 0, 0, 1]                   # only 2's row, [1, 8, 9, 10], brings one: node 1
