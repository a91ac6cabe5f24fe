"""Pins for O-NND, the two-phase NN-Descent oracle (Algorithm 1, sections 3.1.1 and 4).

The sampled iteration is a heuristic with no printed per-round numbers, so it is pinned
through the cases where it is exact by construction, through invariants that hold every
round, through its pieces (merge rule, samples, blocks), and through the qualitative
behaviour the paper reports (section 7.3)."""
import numpy as np
import pytest

import oracle
from paper_2508_08744_amd import inputs


def _check_lists(X, ids, dist, metric=0):
    n, k = ids.shape
    Xd = X.astype(np.float64)
    for v in range(n):
        row = ids[v]
        assert v not in row, "self in list"
        assert len(set(row.tolist())) == k, "duplicate in list"
        keys = list(zip(dist[v].tolist(), row.tolist()))
        assert keys == sorted(keys), "list not sorted by (dist, id)"
    # every stored distance equals an independent fp64 recomputation
    a = Xd[np.repeat(np.arange(n), k)]
    b = Xd[ids.reshape(-1)]
    if metric == 0:
        ref = ((a - b) ** 2).sum(axis=1)
    elif metric == 1:
        ref = -(a * b).sum(axis=1)
    else:
        ref = 1.0 - (a * b).sum(axis=1) / np.sqrt((a * a).sum(axis=1) * (b * b).sum(axis=1))
    np.testing.assert_allclose(dist.reshape(-1), ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("metric", [0, 1, 2])
def test_complete_graph_equals_bruteforce(metric):
    # k = n-1: the random initial lists already hold every other node
    X = inputs.make("C1", n=40, d=6)
    bf_ids, bf_d = oracle.brute_force_knn(X, 39, metric)
    o = oracle.NNDescent(X, 39, metric=metric, seed=3)
    o.init()
    ids, dist, fresh = o.graph()
    assert (ids == bf_ids).all()
    np.testing.assert_array_equal(dist, bf_d)
    assert fresh.all()


@pytest.mark.parametrize("metric", [0, 1, 2])
@pytest.mark.parametrize("cfg", ["C1", "C2"])
def test_exhaustive_round_equals_bruteforce(cfg, metric):
    # one round in which every node meets every other node must give the exact graph,
    # ties included (C2-shaped data is integer valued and has exact distance ties)
    X = inputs.make(cfg, n=180, d=8, comps=3)
    k = 10
    bf_ids, bf_d = oracle.brute_force_knn(X, k, metric)
    o = oracle.NNDescent(X, k, metric=metric, C=0, retain=0, all_block=True, seed=5)
    o.init()
    o.phase1_round()
    ids, dist, _ = o.graph()
    assert (ids == bf_ids).all()
    np.testing.assert_array_equal(dist, bf_d)
    # a second round changes nothing
    assert o.phase1_round() == 0


def test_exhaustive_with_threshold_off_is_identical():
    X = inputs.make("C2", n=150, d=8, comps=3)
    a = oracle.NNDescent(X, 8, C=0, retain=0, all_block=True, seed=5, use_threshold=True)
    b = oracle.NNDescent(X, 8, C=0, retain=0, all_block=True, seed=5, use_threshold=False)
    for o in (a, b):
        o.init()
        o.phase1_round()
    assert (a.graph()[0] == b.graph()[0]).all()


def test_init_lists():
    X = inputs.make("C1", n=500)
    o = oracle.NNDescent(X, 16, seed=42)
    o.init()
    ids, dist, fresh = o.graph()
    _check_lists(X, ids, dist)
    assert fresh.all()
    # the draw is floor(n * u32 / 2^32) of the tagged hash, rejections skipped
    v, got, t = 7, [], 0
    while len(got) < 16:
        c = ((oracle.hash3(42, 1, v, t) >> 32) * 500) >> 32
        t += 1
        if c != v and c not in got:
            got.append(c)
    assert sorted(got) == sorted(ids[v].tolist())
    # ids are spread over the whole range
    hist = np.bincount(ids.reshape(-1), minlength=500)
    assert hist.min() > 0 and hist.max() < 4 * 16
    # another seed gives other lists
    o2 = oracle.NNDescent(X, 16, seed=43)
    o2.init()
    assert (o2.graph()[0] != ids).mean() > 0.9


@pytest.mark.parametrize("params", [
    dict(C=0, retain=0),
    dict(C=32, retain=1, ng_row=2, ng_col=2),
    dict(C=64, retain=1, ng_row=4, ng_col=8),
    dict(C=16, retain=0, S=8, R=8),
])
def test_round_invariants(params):
    X = inputs.make("C1", n=600, d=8)
    k = 12
    o = oracle.NNDescent(X, k, seed=2, **params)
    o.init()
    prev_ids, prev_d, _ = o.graph()
    for r in range(8):
        phase2 = r >= 4
        if r == 4:
            o.begin_phase2()
        upd = o.phase2_round() if phase2 else o.phase1_round()
        ids, dist, fresh = o.graph()
        _check_lists(X, ids, dist)
        # lists only ever improve: entrywise non-increasing distances
        assert (dist <= prev_d).all()
        # updates = number of entries that were not in the list before
        changed = sum(len(set(ids[v].tolist()) - set(prev_ids[v].tolist())) for v in range(len(ids)))
        assert changed == upd == o.counters()["updates"]
        # new arrivals, and only they, carry the flag after a phase-1 round with S >= k
        if not phase2 and params.get("S", k) >= k:
            for v in range(0, len(ids), 37):
                was = set(prev_ids[v].tolist())
                assert [int(i not in was) for i in ids[v]] == fresh[v].tolist()
        prev_ids, prev_d = ids, dist


def test_fixpoint():
    X = inputs.make("C1", n=300, d=4)
    o = oracle.NNDescent(X, 6, C=0, retain=0, seed=1)
    o.init()
    for _ in range(40):
        if o.phase1_round() == 0:
            break
    else:
        pytest.fail("no fixpoint")
    before = o.graph()
    assert o.phase1_round() == 0
    assert o.counters()["pairs"] == 0          # nothing is new any more: no join at all
    after = o.graph()
    assert all((a == b).all() for a, b in zip(before, after))


@pytest.mark.parametrize("params", [dict(C=0, retain=0), dict(C=32, retain=1, ng_row=2, ng_col=4)])
def test_threshold_filter_never_changes_the_result(params):
    # section 4.2: candidates that are not closer than the farthest entry cannot improve the list
    X = inputs.make("C2", n=500, d=16, comps=5)
    a = oracle.NNDescent(X, 10, seed=4, use_threshold=True, **params)
    b = oracle.NNDescent(X, 10, seed=4, use_threshold=False, **params)
    a.init(); b.init()
    for r in range(6):
        if r == 3:
            a.begin_phase2(); b.begin_phase2()
        ua = a.phase2_round() if r >= 3 else a.phase1_round()
        ub = b.phase2_round() if r >= 3 else b.phase1_round()
        assert ua == ub
        ga, gb = a.graph(), b.graph()
        assert (ga[0] == gb[0]).all() and (ga[1] == gb[1]).all() and (ga[2] == gb[2]).all()
    assert a.counters()["offered"] <= b.counters()["offered"]


def _py_merge(self_id, ids, dist, fresh, cid, cd):
    have = set(ids)
    cands = {}
    for i, x in zip(cid, cd):
        if i == self_id or i in have:
            continue
        if i not in cands or x < cands[i]:
            cands[i] = x
    items = [(x, i, f, 0) for i, x, f in zip(ids, dist, fresh)] + [(x, i, 1, 1) for i, x in cands.items()]
    items.sort(key=lambda t: (t[0], t[1]))
    items = items[:len(ids)]
    return [t[1] for t in items], [t[0] for t in items], [t[2] for t in items], sum(t[3] for t in items)


def test_merge_rule():
    rng = np.random.default_rng(3)
    for trial in range(200):
        k = int(rng.integers(1, 12))
        nc = int(rng.integers(0, 20))
        ids = rng.choice(60, size=k, replace=False) + 1
        # few distinct distance values: plenty of exact ties
        dist = np.sort(rng.integers(0, 6, size=k)).astype(np.float64)
        order = np.lexsort((ids, dist))
        ids, dist = ids[order], dist[order]
        fresh = rng.integers(0, 2, size=k)
        cid = rng.integers(0, 61, size=nc)          # includes self (0), repeats and listed ids
        cd = rng.integers(0, 7, size=nc).astype(np.float64)
        # a repeated candidate id always carries the same distance
        for j in range(nc):
            cd[j] = cd[np.nonzero(cid == cid[j])[0][0]]
        want = _py_merge(0, ids.tolist(), dist.tolist(), fresh.tolist(), cid.tolist(), cd.tolist())
        got = oracle.merge_list(0, ids, dist, fresh, cid, cd)
        assert got[0].tolist() == want[0] and got[1].tolist() == want[1]
        assert got[2].tolist() == want[2] and got[3] == want[3]
    # degenerate: no candidates; all candidates already listed
    ids, dist, fresh, ins = oracle.merge_list(9, [1, 2, 3], [1.0, 2.0, 3.0], [0, 1, 0], [], [])
    assert ids.tolist() == [1, 2, 3] and ins == 0 and fresh.tolist() == [0, 1, 0]
    ids, dist, fresh, ins = oracle.merge_list(9, [1, 2, 3], [1.0, 2.0, 3.0], [0, 1, 0], [3, 1, 9], [0.5, 0.5, 0.1])
    assert ids.tolist() == [1, 2, 3] and ins == 0


def test_samples_and_blocks():
    X = inputs.make("C1", n=400, d=8)
    k, S, R = 12, 12, 6
    o = oracle.NNDescent(X, k, S=S, R=R, C=32, seed=8)
    o.init()
    o.phase1_round()
    ids, _, fresh = o.graph()
    o.phase1_sample()                      # samples of the coming round, from the lists above
    n = len(ids)
    new_in = {u: set() for u in range(n)}
    old_in = {u: set() for u in range(n)}
    for v in range(n):
        for u, f in zip(ids[v], fresh[v]):
            (new_in if f else old_in)[int(u)].add(v)
    capped = 0
    for v in range(n):
        NEW, OLD = o.block(v)
        new_fwd = [int(u) for u, f in zip(ids[v], fresh[v]) if f]
        old_fwd = [int(u) for u, f in zip(ids[v], fresh[v]) if not f]
        # forward part first, in list order
        assert NEW[:len(new_fwd)].tolist() == new_fwd
        rev_part = set(NEW[len(new_fwd):].tolist())
        # reverse part: true reverse edges of the right class, not repeated
        assert rev_part <= new_in[v] and not (rev_part & set(new_fwd))
        assert len(rev_part) <= R
        if len(new_in[v]) <= R:
            assert rev_part == new_in[v] - set(new_fwd)
        else:
            capped += 1
        allb = NEW.tolist() + OLD.tolist()
        assert len(set(allb)) == len(allb) and v not in allb
        assert set(OLD.tolist()) <= (set(old_fwd) | old_in[v]) - set(NEW.tolist())
        assert [u for u in old_fwd if u not in set(NEW.tolist())] == OLD[:len([u for u in old_fwd if u not in set(NEW.tolist())])].tolist()
        if len(old_in[v]) <= R:
            assert set(OLD.tolist()) == (set(old_fwd) | old_in[v]) - set(NEW.tolist())
    assert capped > 0, "test should exercise the reverse cap"


def test_reverse_cap_is_a_uniform_subset():
    # a star: every node lists node 0, so node 0 has n-1 reverse arrivals and keeps R of them
    n, k, R = 65, 3, 8
    X = inputs.make("C1", n=n, d=3)
    ids = np.zeros((n, k), dtype=np.int32)
    for v in range(n):
        others = [u for u in range(1, n) if u != v]
        ids[v] = ([0] + others[:k - 1]) if v != 0 else others[:k]
    dist = np.array([[oracle.distance(X, 0, v, int(u)) for u in ids[v]] for v in range(n)])
    order = np.lexsort((ids, dist), axis=1)
    ids = np.take_along_axis(ids, order, axis=1)
    dist = np.take_along_axis(dist, order, axis=1)
    hits = np.zeros(n)
    trials = 400
    for seed in range(trials):
        o = oracle.NNDescent(X, k, S=k, R=R, C=32, seed=seed)
        o.set_graph(ids, dist, np.ones_like(ids, dtype=np.uint8))
        o.phase1_sample()
        NEW, OLD = o.block(0)
        assert len(OLD) == 0
        assert NEW[:k].tolist() == ids[0].tolist()
        rev = NEW[k:].tolist()
        # R arrivals are drawn; those already in the forward part are not repeated
        assert R - k <= len(rev) <= R and not set(rev) & set(ids[0].tolist())
        for u in rev:
            hits[u] += 1
    # each node outside the anchor's own list is chosen about equally often: R/(n-1) of the time
    outside = [u for u in range(1, n) if u not in ids[0].tolist()]
    freq = hits[outside] / trials
    assert abs(freq.mean() - R / (n - 1)) < 0.01
    assert freq.max() < 2.0 * R / (n - 1) and freq.min() > 0.4 * R / (n - 1)


def test_two_phase_behaviour():
    # section 7.3: phase 1 alone slows down at high recall, phase 2 keeps improving;
    # recall >= 0.95 is reached within 16 rounds in total
    X = inputs.make("C1", n=3000)
    k = 16
    truth, _ = oracle.brute_force_knn(X, k)
    kw = dict(C=32, retain=1, ng_row=2, ng_col=2, seed=1)

    def recall_after(it1, it2):
        o = oracle.NNDescent(X, k, **kw)
        o.run(it1, it2)
        return oracle.recall(o.graph()[0], truth)

    only1 = recall_after(10, 0)
    both = recall_after(5, 5)
    assert both > only1
    assert both >= 0.95
    assert recall_after(8, 8) >= both - 1e-3
    # an untouched random graph is near zero recall
    assert recall_after(0, 0) < 0.05


def test_early_stop():
    X = inputs.make("C1", n=1000)
    o = oracle.NNDescent(X, 16, C=32, seed=1)
    r1, r2 = o.run(16, 16, delta=0.01)
    assert 1 <= r1 < 16 and 1 <= r2 < 16
    o2 = oracle.NNDescent(X, 16, C=32, seed=1)
    assert o2.run(3, 2, delta=0.0) == (3, 2)


@pytest.mark.parametrize("retain", [0, 1])
def test_join_pair_count_is_new_new_plus_new_old(retain):
    # 3.1.1 step (2): distances between new-new and new-old pairs, never old-old
    X = inputs.make("C1", n=300, d=8)
    k = 10
    o = oracle.NNDescent(X, k, S=k, R=5, C=32, retain=retain, seed=6)
    o.init()
    o.phase1_round()
    o.phase1_round()
    state = o.graph()
    o.phase1_sample()
    want = 0
    for v in range(300):
        NEW, OLD = o.block(v)
        want += len(NEW) * (len(NEW) - 1) // 2 + len(NEW) * len(OLD)
    o.set_graph(*state)
    o.phase1_round()
    assert o.counters()["pairs"] == want > 0


def test_new_old_pair_reaches_both_lists():
    # anchor 0 lists a=1 (new) and b=2 (old); 1 and 2 are each other's nearest point but do
    # not list each other yet: one round must introduce them to each other, in both directions
    X = np.array([[0.0], [10.0], [10.5], [100.0], [200.0], [300.0], [400.0]], dtype=np.float32)
    n, k = len(X), 2
    ids = np.array([[1, 2], [3, 4], [3, 4], [4, 5], [3, 5], [4, 6], [5, 4]], dtype=np.int32)
    dist = np.array([[oracle.distance(X, 0, v, int(u)) for u in ids[v]] for v in range(n)])
    order = np.lexsort((ids, dist), axis=1)
    ids, dist = np.take_along_axis(ids, order, 1), np.take_along_axis(dist, order, 1)
    fresh = np.zeros_like(ids, dtype=np.uint8)
    fresh[0] = (ids[0] == 1)                      # only the edge 0 -> 1 is new
    o = oracle.NNDescent(X, k, S=k, R=4, C=8, seed=1)
    o.set_graph(ids, dist, fresh)
    upd = o.phase1_round()
    g, gd, gf = o.graph()
    assert 2 in g[1] and 1 in g[2]
    assert gd[1][0] == pytest.approx(0.25) and gd[2][0] == pytest.approx(0.25)
    # pairs: (1,2) at anchor 0, and at anchor 1 its new reverse arrival 0 against 1's two old entries
    # (node 0 is closer to 3 than 3's farthest entry, so that pair is a third update)
    assert o.counters()["pairs"] == 3 and upd == 3 and 0 in g[3]
    # the sampled new edge is old now, the two arrivals are new
    assert gf[0].tolist() == [0, 0]
    assert gf[1][g[1].tolist().index(2)] == 1 and gf[2][g[2].tolist().index(1)] == 1


def test_phase2_semantics():
    # the phase-2 loop of Algorithm 1 and the non-revisitation rule of section 4.1
    X = inputs.make("C1", n=500, d=8)
    k, m = 10, 2
    o = oracle.NNDescent(X, k, C=32, m=m, seed=3)
    o.init()
    for _ in range(2):
        o.phase1_round()
    o.begin_phase2()
    assert o.graph()[2].all()                    # everything unvisited at the switch
    for r in range(4):
        ids0, d0, f0 = o.graph()
        o.phase2_round()
        ids1, d1, f1 = o.graph()
        measured = 0
        for v in range(500):
            expanded = [int(u) for u, f in zip(ids0[v], f0[v]) if f][:m]
            pool = set()
            for u in expanded:
                pool |= set(ids0[u].tolist())    # lists as they stood when the round began
            measured += len(pool - {v} - set(ids0[v].tolist()))      # each once; never v itself or a listed node
            arrived = set(ids1[v].tolist()) - set(ids0[v].tolist())
            assert arrived <= pool - {v}
            # the list is exactly the best k of (old list + pool)
            cand = sorted((oracle.distance(X, 0, v, c), c) for c in (pool | set(ids0[v].tolist())) - {v})[:k]
            assert [c for _, c in cand] == ids1[v].tolist()
            # expanded entries are visited now, arrivals are unvisited, the rest keeps its mark
            for u, f in zip(ids1[v], f1[v]):
                u = int(u)
                if u in arrived:
                    assert f == 1
                elif u in expanded:
                    assert f == 0
                else:
                    assert f == f0[v][ids0[v].tolist().index(u)]
        assert o.counters()["pairs"] == measured


def test_candidate_slots_spread_evenly():
    # One (target, anchor) pair owns one line of 8 slots: its opponent groups land in distinct
    # words of that line.  Over many anchors all C slots of a target are used about equally,
    # and two anchors that share a line at one target or round do not share it at all of them.
    for C in (16, 64, 128, 256):
        counts = np.zeros(C)
        for v in range(4000):
            ss = [oracle.slot_of(7, 3, 123, v, g, C) for g in range(8)]
            assert all(0 <= s < C for s in ss)
            assert len({s // 8 for s in ss}) == 1 and len(set(ss)) == 8
            assert [(s - ss[0]) % 8 for s in ss] == list(range(8))     # consecutive words, rotated
            counts[ss[v % 8]] += 1                                     # one group per anchor, all groups in turn
        mean = 4000 / C                              # counts behave like Poisson(mean)
        assert counts.min() > mean - 5 * mean ** 0.5 and counts.max() < mean + 5 * mean ** 0.5
    same = sum(oracle.slot_of(7, r, t, 10, 0, 64) // 8 == oracle.slot_of(7, r, t, 77, 0, 64) // 8
               for r in range(20) for t in range(50))
    assert 80 <= same <= 175        # about 1000 / 8 lines by chance


@pytest.mark.parametrize("tile,ngr,ngc", [(2, 2, 2), (1, 2, 4), (3, 4, 2), (16, 4, 8)])
def test_retention_keeps_one_candidate_per_target_and_group_of_opposite_positions(tile, ngr, ngc):
    """Section 4.2 retention, counted: with the threshold off every pair passes, so a row member keeps one
    candidate for every group of column positions it meets, a column member one for every group of row
    positions: the number of candidates handed over follows from the block sizes alone."""
    X = inputs.make("C1", n=200, d=8)
    k = 10
    o = oracle.NNDescent(X, k, S=k, R=6, C=32, retain=1, tile=tile, ng_row=ngr, ng_col=ngc, seed=3, use_threshold=False)
    o.init()
    o.phase1_round()
    state = o.graph()
    o.phase1_sample()
    want = 0
    for v in range(200):
        NEW, OLD = o.block(v)
        nN, nT = len(NEW), len(NEW) + len(OLD)
        if nN == 0 or nT < 2:
            continue
        for a in range(nN):                                   # row member a meets the columns behind it
            want += len({(b // tile) % ngc for b in range(a + 1, nT)})
        for b in range(nT):                                   # column member b meets the rows in front of it
            want += len({(a // tile) % ngr for a in range(min(b, nN))})
    o.set_graph(*state)
    o.phase1_round()
    assert o.counters()["offered"] == want > 0


def test_forward_sample_takes_the_first_S_of_each_class():
    """Section 3.1.1 sampling with S < k: the block of v begins with its first S new entries in list order,
    reverse edges come from sampled edges only, and only the sampled new entries turn old."""
    X = inputs.make("C1", n=300, d=8)
    k, S, R = 12, 3, 24
    o = oracle.NNDescent(X, k, S=S, R=R, C=32, seed=8)
    o.init()
    o.phase1_round()
    ids, dist, fresh = o.graph()
    o.phase1_sample()
    first_new = [[int(u) for u, f in zip(ids[v], fresh[v]) if f][:S] for v in range(300)]
    first_old = [[int(u) for u, f in zip(ids[v], fresh[v]) if not f][:S] for v in range(300)]
    more_new = 0
    for v in range(300):
        NEW, OLD = o.block(v)
        more_new += int(fresh[v].sum() > S)
        assert NEW[:len(first_new[v])].tolist() == first_new[v]
        rev_new = set(NEW[len(first_new[v]):].tolist())
        assert rev_new == {u for u in range(300) if v in first_new[u]} - set(first_new[v])      # R is large: no cap
        assert set(OLD.tolist()) == (set(first_old[v]) | {u for u in range(300) if v in first_old[u]}) - set(NEW.tolist())
    assert more_new > 100, "lists should hold more than S new entries"
    o.phase1_round()
    ids2, _, fresh2 = o.graph()
    for v in range(300):
        now = dict(zip(ids2[v].tolist(), fresh2[v].tolist()))
        for u, f in zip(ids[v].tolist(), fresh[v].tolist()):
            if u in now and f:
                assert now[u] == (0 if u in first_new[v] else 1)       # sampled: old now; not sampled: still new


# ---------------------------------------------------------------------------------------------
# The two readings added for a bounded hand-over: a node the target's list holds is no candidate
# where the pair is met (exclude_listed), and a round carried out in parts with an update after
# each.  For the plain method (every pair offered, unbounded candidate lists) neither can change a
# list: the update drops a listed node anyway, and a candidate that a tightened threshold turns
# away could not have stayed.  With retention both matter; there the oracle is checked against a
# round written out in Python on a small input.
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,n,k", [("C1", 700, 8), ("C2", 600, 12)])
def test_plain_method_is_blind_to_exclusion_and_parts(cfg, n, k):
    X = inputs.make(cfg, n=n, d=8, comps=4)
    ref = oracle.NNDescent(X, k, seed=9)
    variants = [oracle.NNDescent(X, k, seed=9, exclude_listed=True),
                oracle.NNDescent(X, k, seed=9, parts=3),
                oracle.NNDescent(X, k, seed=9, parts=4, exclude_listed=True)]
    for o in [ref] + variants:
        o.init()
    for r in range(4):
        ref.phase1_round()
        want = ref.graph()
        offered = ref.counters()["offered"]
        for j, o in enumerate(variants):
            o.phase1_round()
            got = o.graph()
            assert all((a == b).all() for a, b in zip(got, want)), (r, j)
            c = o.counters()
            assert c["pairs"] == ref.counters()["pairs"]
            assert c["offered"] <= offered, "fewer nodes are offered, never more"
            if j == 0:
                assert c["updates"] == ref.counters()["updates"]        # one update per round: the same entries change
            else:
                assert c["updates"] >= ref.counters()["updates"]        # an entry may come and go inside one round
    ref.begin_phase2()
    for o in variants:
        o.begin_phase2()
    ref.phase2_round()
    for o in variants:
        o.phase2_round()
        assert all((a == b).all() for a, b in zip(o.graph(), ref.graph()))


def _python_round(X, ids, dist, fresh, blocks, k, tile, ng, exclude, parts, C=0, seed=0, rnd=0):
    """One phase-1 round written out: blocks fixed, sampled entries old, then for each part the join of its anchors
    with per (member, group of opposite positions) retention of the closest admissible node, and the update.
    C > 0: a node has C candidate slots; what a block keeps for it goes to slot_of(...) and the closer one stays."""
    n = len(X)
    Xd = X.astype(np.float64)
    lists = [[(dist[v, j], int(ids[v, j]), 0 if sampled else int(fresh[v, j])) for j, sampled in enumerate(smp)]
             for v, smp in enumerate(blocks["sampled"])]
    for p in range(parts):
        cands = [dict() for _ in range(n)]           # target -> {(anchor, row or column node, group): (dist, id)}
        for v in range(p, n, parts):
            N, O = blocks["blocks"][v]
            mem = list(N) + list(O)
            if len(N) == 0 or len(mem) < 2:
                continue
            for a in range(len(N)):
                for b in range(a + 1, len(mem)):
                    t, c = mem[a], mem[b]
                    dd = float(((Xd[t] - Xd[c]) ** 2).sum())
                    for role, (tgt, cnd, opp) in enumerate(((t, c, b), (c, t, a))):       # the row node's turn, the column node's
                        L = lists[tgt]
                        if exclude and any(e[1] == cnd for e in L):
                            continue
                        if not (dd, cnd) < (L[-1][0], L[-1][1]):
                            continue
                        key = (v, role, (opp // tile) % ng)
                        if key not in cands[tgt] or (dd, cnd) < cands[tgt][key]:
                            cands[tgt][key] = (dd, cnd)
        for t in range(n):
            L = lists[t]
            have = {e[1] for e in L}
            kept = cands[t]
            if C > 0:
                kept = {}
                for (v, role, g), cand in cands[t].items():
                    slot = oracle.slot_of(seed, rnd, t, v, g, C)
                    if slot not in kept or cand < kept[slot]:
                        kept[slot] = cand
            new = sorted(set(kept.values()))
            for dd, c in new:
                if c == t or c in have:
                    continue
                have.add(c)
                L.append((dd, c, 1))
            L.sort(key=lambda e: (e[0], e[1]))
            del L[k:]
    return lists


@pytest.mark.parametrize("exclude", [False, True])
@pytest.mark.parametrize("parts,C", [(1, 0), (3, 0), (3, 16)])
def test_round_with_retention_exclusion_and_parts_against_a_python_round(exclude, parts, C):
    n, k, tile, ng = 150, 6, 4, 8
    X = inputs.make("C2", n=n, d=6, comps=3)          # integer valued: distances exact either way, ties occur
    X[5:10] = X[0:5]                                    # and a few points twice: distance 0 between them
    o = oracle.NNDescent(X, k, S=k, R=5, C=C, retain=1, tile=tile, ng_row=ng, ng_col=ng, seed=4,
                         exclude_listed=exclude, parts=parts)
    o.init()
    for r in range(3):
        ids, dist, fresh = o.graph()
        o.phase1_sample()
        blk = [o.block(v) for v in range(n)]
        # sampled = the first S new entries of every list (S = k: every new entry)
        sampled = [[bool(fresh[v, j]) for j in range(k)] for v in range(n)]
        want = _python_round(X, ids, dist, fresh, dict(blocks=blk, sampled=sampled), k, tile, ng, exclude, parts, C=C, seed=4, rnd=r)
        o.phase1_round()
        gi, gd, gf = o.graph()
        for v in range(n):
            assert [e[1] for e in want[v]] == gi[v].tolist(), (r, v)
            assert [e[0] for e in want[v]] == gd[v].tolist(), (r, v)
            assert [e[2] for e in want[v]] == gf[v].tolist(), (r, v)


def test_exclusion_lets_the_next_closest_node_through():
    """Hand-made: with one retention group a member keeps the closest of the nodes behind it in its block.  Nodes 0, 1, 2
    meet only in the block of node 7, in this order.  Node 1 is the closest to node 0 and sits in 0's list already: without
    exclude_listed it takes the one place and the update throws it away; with it, node 2 reaches node 0."""
    X = np.array([[0.0], [1.0], [2.5], [100.0], [101.0], [103.0], [106.0], [-50.0]], dtype=np.float32)
    n, k = len(X), 3
    lists = [[1, 3, 4], [0, 3, 4], [3, 4, 5], [4, 5, 6], [3, 5, 6], [4, 3, 6], [5, 4, 3], [0, 1, 2]]

    def run(exclude):
        o = oracle.NNDescent(X, k, S=k, R=0, C=0, retain=1, tile=64, ng_row=1, ng_col=1, seed=1, exclude_listed=exclude)
        o.init()
        ids = np.array(lists, dtype=np.int32)
        dist = np.array([[float((X[v, 0] - X[c, 0]) ** 2) for c in ids[v]] for v in range(n)])
        assert (np.diff(dist, axis=1) >= 0).all(), "the hand-made rows are in list order (the one tie is in id order)"
        o.set_graph(ids, dist, np.ones((n, k), dtype=np.uint8))
        o.phase1_sample()
        assert [b.tolist() for b in o.block(7)] == [[0, 1, 2], []]
        assert all(not ({0, 2} <= set(o.block(v)[0].tolist())) for v in range(7)), "0 and 2 meet in one block only"
        o.phase1_round()
        return o.graph()[0]

    without, with_ = run(False), run(True)
    assert without[0].tolist() == [1, 3, 4], "node 1, already listed, took node 2's place"
    assert with_[0].tolist() == [1, 2, 3]
    # the other two nodes of the block fare alike either way: 1 gets 2 (its place as a row node is its own), 2 gets 1
    for g in (without, with_):
        assert g[1].tolist() == [0, 2, 3] and g[2].tolist() == [1, 3, 4]
