"""GPU parity: the HIP path, called through the C boundary, against the CPU oracle.

Integer-valued inputs (the C2 recipe: byte-valued features) make every fp32 operation of
the HIP path exact, so there the two must agree bit for bit after every step.  On real-valued
inputs the decisions are taken in different precisions (fp32 Gram form vs fp64), so the
comparison is statistical: recall within 0.005 of the oracle's at equal rounds, every reported
distance within 1e-4 relative of an fp64 recomputation, lists sorted, duplicate-free, self-free.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu

REL_TOL = 1e-4          # spec tolerance for reported distances
RECALL_TOL = 0.005      # spec tolerance for recall against the oracle


def _oracle_for(X, prm, metric=0):
    return oracle.NNDescent(X, prm.k, metric=metric, **oracle.device_model(prm))


def _same(gpu_graph, oracle_graph):
    gi, gd, gf = [t.cpu().numpy() for t in gpu_graph]
    oi, od, of = oracle_graph
    return (gi == oi).all() and (gd.astype(np.float64) == od).all() and (gf == of).all()


def _ref_dist(X, rows, ids, metric):
    Xd = X.astype(np.float64)
    a = Xd[rows][:, None, :]
    b = Xd[ids]
    if metric == 0:
        return ((a - b) ** 2).sum(-1)
    dot = (a * b).sum(-1)
    if metric == 1:
        return -dot
    return 1.0 - dot / np.sqrt((a * a).sum(-1) * (b * b).sum(-1))


def _check_properties(X, ids, dist, metric=0, rows=None):
    n, k = ids.shape
    rows = np.arange(n) if rows is None else rows
    assert (ids >= 0).all() and (ids < len(X)).all()
    assert (ids != rows[:, None]).all(), "self in list"
    srt = np.sort(ids, axis=1)
    assert (srt[:, 1:] != srt[:, :-1]).all(), "duplicate id in a list"
    assert (dist[:, 1:] >= dist[:, :-1]).all(), "list not sorted by distance"
    ties = dist[:, 1:] == dist[:, :-1]
    assert (ids[:, 1:][ties] > ids[:, :-1][ties]).all(), "equal distances not ordered by id"
    ref = _ref_dist(X, rows, ids, metric)
    scale = 1e-6 * float((X.astype(np.float64) ** 2).sum(1).mean())
    rel = np.abs(dist - ref) / np.maximum(np.abs(ref), scale)
    assert rel.max() <= REL_TOL, rel.max()


@pytest.mark.parametrize("d", [4, 32, 100, 128, 200, 960])
def test_join_distance_tile(d):
    """The LDS/MFMA distance core on explicit blocks, ragged shapes included."""
    n = 700
    rng = np.random.default_rng(d)
    X = rng.standard_normal((n, d)).astype(np.float32)
    prm = knn.default_params(16, 4)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    shapes = [(64, 64), (1, 1), (17, 30), (64, 0), (5, 0), (33, 95), (16, 16), (2, 0), (1, 127), (48, 49)]
    blk = np.zeros((len(shapes), 128), dtype=np.int32)
    sizes = np.zeros((len(shapes), 2), dtype=np.int32)
    for i, (a, o) in enumerate(shapes):
        blk[i, :a + o] = rng.choice(n, size=a + o, replace=False)
        sizes[i] = (a, o)
    out = b.join_distances(torch.from_numpy(blk), torch.from_numpy(sizes)).cpu().numpy()
    Xd = X.astype(np.float64)
    for i, (a, o) in enumerate(shapes):
        P = Xd[blk[i, :a + o]]
        ref = ((P[:, None, :] - P[None, :, :]) ** 2).sum(-1)
        used = np.zeros((64, 128), dtype=bool)
        for r in range(a):
            used[r, r + 1:a + o] = True
        got = out[i][:a, :a + o]
        m = used[:a, :a + o]
        # norm-plus-Gram form in fp32: absolute error scales with the norms
        tol = 4e-6 * (Xd ** 2).sum(1).max()
        assert np.abs(got[m] - ref[:a][m]).max() <= tol
        assert np.isnan(out[i][~used]).all(), "wrote outside the needed pairs"
    b.close()


def test_join_distance_rejects_bad_blocks():
    X = torch.zeros((100, 8), device="cuda")
    b = knn.Builder(X, knn.default_params(4, 2))
    blk = torch.zeros((1, 128), dtype=torch.int32)
    for sizes in ([65, 0], [10, 119], [-1, 3]):
        with pytest.raises(knn.TagoreError):
            b.join_distances(blk, torch.tensor([sizes], dtype=torch.int32))
    blk[0, 1] = 100
    with pytest.raises(knn.TagoreError):
        b.join_distances(blk, torch.tensor([[2, 0]], dtype=torch.int32))
    b.close()


@pytest.mark.parametrize("n,d,k,kw", [(2000, 64, 32, dict(parts=4)), (700, 16, 48, dict(parts=2, R=32)), (500, 8, 64, dict(parts=1)),
                                      (900, 24, 10, dict(parts=8, S=4, R=20))])
def test_block_adjacency_words_are_the_lists(n, d, k, kw):
    """What the join is told about a block, "the node at position x is in position p's list already", against the
    definition, for every member of every block (blocks of up to 128 members, ids that share a table slot)."""
    X = inputs.make("C2", n=n, d=d, comps=4)
    prm = knn.default_params(k, 6, seed=11, **kw)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    b.init()
    for r in range(3):
        blk, sizes = b.sample_blocks()
        adj = b.block_adjacency()
        blk, sizes = blk.cpu().numpy(), sizes.cpu().numpy()
        adj = adj.cpu().numpy().view(np.uint32)
        ids = b.graph()[0].cpu().numpy()
        for v in range(n):
            nT = int(sizes[v].sum())
            if sizes[v, 0] == 0 or nT < 2:
                assert not adj[v].any()
                continue
            mem = blk[v, :nT]
            pos = {int(x): i for i, x in enumerate(mem)}
            want = np.zeros((128, 4), dtype=np.uint32)
            for p in range(nT):
                for c in ids[mem[p]]:
                    x = pos.get(int(c))
                    if x is not None:
                        want[p, x >> 5] |= np.uint32(1 << (x & 31))
            assert (adj[v] == want).all(), (r, v)
        b.phase1_round()
    b.close()


STEPWISE = [
    # n, d, k, overrides: several tiles, ragged tails, odd d (padded rows), small and large caps
    (3000, 64, 32, dict(C=64, parts=4)),
    (2500, 100, 16, dict(C=32, parts=1, R=8)),
    (1200, 30, 10, dict(C=16, parts=2, S=6, R=20)),
    (1500, 132, 32, dict(C=128, parts=8)),
    (900, 7, 48, dict(C=64, parts=2, R=32)),
    (400, 16, 64, dict(C=128, parts=4, m=3)),
    (1000, 256, 32, dict(C=256)),          # long rows: the workgroup join with 128-column slabs
    (1400, 128, 32, dict(C=256)),          # the bench shape of rows and slots
]


@pytest.mark.parametrize("n,d,k,kw", STEPWISE)
def test_every_step_identical_to_oracle(n, d, k, kw):
    """Algorithm 1 step by step on integer-valued data: blocks, lists, marks and update counts."""
    X = inputs.make("C2", n=n, d=d, comps=max(2, n // 500))
    prm = knn.default_params(k, 8, seed=5, **kw)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    b.init()
    o.init()
    assert _same(b.graph(), o.graph()), "initial lists"
    for r in range(4):
        blk, sizes = b.sample_blocks()
        blk, sizes = blk.cpu().numpy(), sizes.cpu().numpy()
        o.phase1_sample()
        for v in range(n):
            N, O = o.block(v)
            assert sizes[v, 0] == len(N) and sizes[v, 1] == len(O), (r, v)
            assert (blk[v, :len(N)] == N).all() and (blk[v, len(N):len(N) + len(O)] == O).all(), (r, v)
            assert (blk[v, len(N) + len(O):] == -1).all()
        assert b.phase1_round() == o.phase1_round(), "update count, phase 1 round %d" % r
        assert _same(b.graph(), o.graph()), "lists after phase 1 round %d" % r
    b.begin_phase2()
    o.begin_phase2()
    assert _same(b.graph(), o.graph())
    for r in range(4):
        assert b.phase2_round() == o.phase2_round(), "update count, phase 2 round %d" % r
        assert _same(b.graph(), o.graph()), "lists after phase 2 round %d" % r
    ids, dist = b.finalize()
    oi, od, _ = o.graph()
    assert (ids.cpu().numpy() == oi).all() and (dist.cpu().numpy().astype(np.float64) == od).all()
    st = b.stats()
    assert st["rounds_phase1"] == 4 and st["rounds_phase2"] == 4
    b.close()


def test_join_statistics_count_the_needed_pairs():
    X = inputs.make("C2", n=2000, d=32, comps=4)
    prm = knn.default_params(16, 6, seed=2)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    b.init(); o.init()
    for r in range(3):
        b.phase1_round(); o.phase1_round()
        assert b.stats()["join_pairs"][r] == o.counters()["pairs"]
    b.close()


@pytest.mark.parametrize("k,m", [(16, 2), (24, 3), (40, 2)])
def test_phase2_counts_every_candidate_once(k, m):
    """Algorithm 1, phase-2 loop: the candidates of a round are the ids listed by the m expanded
    neighbours that are neither v, nor in G[v], nor met before in the same round."""
    X = inputs.make("C2", n=2000, d=32, comps=4)
    prm = knn.default_params(k, 6, seed=2, m=m)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    b.init(); o.init()
    for r in range(2):
        b.phase1_round(); o.phase1_round()
    b.begin_phase2(); o.begin_phase2()
    for r in range(2, 5):
        assert b.phase2_round() == o.phase2_round()
        assert b.stats()["join_pairs"][r] == o.counters()["pairs"], r
        assert _same(b.graph(), o.graph())
    b.close()


@pytest.mark.parametrize("metric", ["l2", "ip", "cosine"])
@pytest.mark.parametrize("d", [40, 200])
def test_screening_never_changes_the_graph(metric, d):
    """The 8-bit lower bound of phase 2 may only drop candidates that could not enter the list:
    on real-valued data of mixed sign and scale the graph with screening equals the one without."""
    rng = np.random.default_rng(77 + d)
    n, k = 6000, 20
    centres = rng.normal(size=(12, d)) * 3.0
    X = (centres[rng.integers(0, 12, n)] + rng.normal(size=(n, d)) * rng.uniform(0.2, 1.5, size=(n, 1))).astype(np.float32)
    X[: n // 3] += 5.0                         # a shifted part: codes with a large offset
    X[n // 3: n // 2] *= 1e-3                  # and a tiny-scale part
    Xg = torch.from_numpy(X).cuda()
    out = []
    for screen in (1, 0):
        prm = knn.default_params(k, 8, metric=metric, seed=9, screen=screen)
        ids, dist, st = knn.knn_build_ex(Xg, prm)
        out.append((ids.cpu().numpy(), dist.cpu().numpy(), st))
    assert (out[0][0] == out[1][0]).all() and (out[0][1] == out[1][1]).all()
    assert out[0][2]["updates"] == out[1][2]["updates"]


@pytest.mark.parametrize("metric", ["l2", "ip", "cosine"])
def test_screening_never_changes_the_graph_where_it_drops_most(metric):
    """Byte-valued data are their own codes, so the bound is as tight as it gets and nearly every candidate is
    dropped on it: the graph must still be the one obtained by measuring every candidate, for all three metrics."""
    X = inputs.make("C2", n=8000, d=100, comps=16)
    Xg = torch.from_numpy(X).cuda()
    out = []
    for screen in (1, 0):
        prm = knn.default_params(24, 8, metric=metric, seed=5, screen=screen)
        ids, dist, st = knn.knn_build_ex(Xg, prm)
        out.append((ids.cpu().numpy(), dist.cpu().numpy(), st))
    assert (out[0][0] == out[1][0]).all() and (out[0][1] == out[1][1]).all()
    assert out[0][2]["updates"] == out[1][2]["updates"]
    r1 = out[0][2]["rounds_phase1"]
    pairs, vecs = out[0][2]["join_pairs"][r1:], out[0][2]["join_vectors"][r1:]
    assert sum(vecs) < 0.5 * sum(pairs), (pairs, vecs)          # the screen did drop candidates


def test_screening_switches_itself_off_where_it_does_not_pay():
    """Byte-valued data: few candidates reach the fp32 evaluation in every phase-2 round.  Real-valued
    data in high dimension: most pass the 8-bit bound in the first screened round, and from the second
    round on every candidate is measured directly (fp32 vectors == candidates)."""
    Xi = inputs.make("C2", n=20000, d=128, comps=20)
    Xr = inputs.make("C4", n=20000, comps=20)
    for X, metric, pays in ((Xi, "l2", True), (Xr, "cosine", False)):
        prm = knn.default_params(16, 8, metric=metric, seed=3)
        _, _, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        r1 = st["rounds_phase1"]
        pairs, vecs = st["join_pairs"][r1:], st["join_vectors"][r1:]
        if pays:
            assert all(v < 0.25 * p for v, p in zip(vecs, pairs)), (pairs, vecs)
        else:
            assert vecs[0] > 0.5 * pairs[0] and vecs[0] < pairs[0]
            assert vecs[1:] == pairs[1:], (pairs, vecs)


@pytest.mark.parametrize("iters", [1, 6, 9])
def test_whole_build_identical_to_oracle(iters):
    X = inputs.make("C2", n=2000, d=48, comps=4)
    prm = knn.default_params(24, iters, seed=11)
    ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    assert o.run(prm.it1, prm.it2) == (st["rounds_phase1"], st["rounds_phase2"])
    oi, od, _ = o.graph()
    assert (ids.cpu().numpy() == oi).all()
    assert (dist.cpu().numpy().astype(np.float64) == od).all()


def test_plain_entry_point_and_early_stop():
    X = inputs.make("C2", n=3000, d=32, comps=6)
    Xg = torch.from_numpy(X).cuda()
    ids, dist = knn.knn_build(Xg, 16, "l2", iters=6, seed=4)
    prm = knn.default_params(16, 6, seed=4)
    o = _oracle_for(X, prm)
    o.run(prm.it1, prm.it2)
    assert (ids.cpu().numpy() == o.graph()[0]).all()
    # iters <= 0: up to 16 rounds, each phase stops once a round changes < 0.1 % of the entries
    ids0, _ = knn.knn_build(Xg, 16, "l2", iters=0, seed=4)
    prm0 = knn.default_params(16, 0, seed=4)
    o0 = _oracle_for(X, prm0)
    o0.run(prm0.it1, prm0.it2, delta=float(np.float32(prm0.delta)))
    assert (ids0.cpu().numpy() == o0.graph()[0]).all()
    truth, _ = oracle.brute_force_knn(X, 16)
    assert oracle.recall(ids0.cpu().numpy(), truth) > 0.97
    # a coarser threshold that is certain to end both phases early, at the same rounds as the oracle
    prm1 = knn.default_params(16, 0, seed=4, delta=0.02)
    ids1, _, st1 = knn.knn_build_ex(Xg, prm1)
    o1 = _oracle_for(X, prm1)
    r1, r2 = o1.run(prm1.it1, prm1.it2, delta=float(np.float32(prm1.delta)))
    assert r1 < prm1.it1 and r2 < prm1.it2
    assert (r1, r2) == (st1["rounds_phase1"], st1["rounds_phase2"])
    assert (ids1.cpu().numpy() == o1.graph()[0]).all()


@pytest.mark.parametrize("cfg,metric", [("C1", "l2"), ("C4", "cosine"), ("C4", "ip"), ("C3", "l2")])
def test_statistical_parity_on_real_valued_data(cfg, metric):
    """Recall within 0.005 of the oracle's at equal rounds (mean over 3 seeds); reported
    distances within 1e-4 relative of fp64; lists well-formed."""
    sizes = {"C1": dict(n=6000), "C4": dict(n=5000, comps=10), "C3": dict(n=3000, d=200, comps=6)}[cfg]
    X = inputs.make(cfg, **sizes)
    k = 16
    mcode = knn.METRICS[metric]
    truth, _ = oracle.brute_force_knn(X, k, mcode)
    gaps = []
    for seed in (1, 2, 3):
        prm = knn.default_params(k, 6, metric=metric, seed=seed, C=32)
        ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        ids, dist = ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64)
        _check_properties(X, ids, dist, mcode)
        o = _oracle_for(X, prm, mcode)
        o.run(prm.it1, prm.it2)
        r_gpu = oracle.recall(ids, truth)
        r_cpu = oracle.recall(o.graph()[0], truth)
        gaps.append(r_gpu - r_cpu)
        assert r_gpu > 0.85
    assert np.mean(gaps) >= -RECALL_TOL, gaps


@pytest.mark.parametrize("cfg,n", [("C1", 10000), ("C2", 20000)])
def test_recall_against_the_plain_oracle(cfg, n):
    """The plain entry point against the plain method (O-NND's reference mode: every evaluated pair offered to both
    nodes, unbounded candidate lists, one list update per round; section 3.1.1, Algorithm 1) at equal rounds:
    recall within 0.005."""
    c = inputs.CONFIGS[cfg]
    k, mcode = c["k"], knn.METRICS[c["metric"]]
    X = inputs.make(cfg, n=n)
    rows = inputs.sample_rows(n, 2000, seed=4)
    truth, _ = oracle.brute_force_knn(X, k, mcode, rows)
    Xg = torch.from_numpy(X).cuda()
    gaps = []
    for seed in (1, 2):
        ids, _ = knn.knn_build(Xg, k, c["metric"], iters=4, seed=seed)
        prm = knn.default_params(k, 4, metric=c["metric"], seed=seed)
        plain = oracle.NNDescent(X, k, mcode, S=prm.S, R=prm.R, m=prm.m, seed=seed)
        plain.run(prm.it1, prm.it2)
        r_gpu = oracle.recall(ids.cpu().numpy()[rows], truth)
        r_plain = oracle.recall(plain.graph()[0][rows], truth)
        assert r_plain > 0.95
        gaps.append(r_gpu - r_plain)
    assert min(gaps) >= -RECALL_TOL, gaps


def test_whole_build_identical_to_oracle_at_mid_size():
    """Every step of a build of 50 000 points (d = 128, k = 32: the C2 recipe, wave and workgroup kernels, many
    blocks per slot line) against the model of its hand-over: ids and distances bit for bit."""
    n, k = 50000, 32
    X = inputs.make("C2", n=n)
    prm = knn.default_params(k, 0, seed=5, it1=2, it2=1, delta=0.0)
    ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    assert o.run(prm.it1, prm.it2) == (st["rounds_phase1"], st["rounds_phase2"])
    oi, od, _ = o.graph()
    assert (ids.cpu().numpy() == oi).all()
    assert (dist.cpu().numpy().astype(np.float64) == od).all()


def test_phase1_lists_keep_their_invariants_without_finalize():
    X = inputs.make("C1", n=4000)
    prm = knn.default_params(16, 8, seed=3)
    b = knn.Builder(torch.from_numpy(X).cuda(), prm)
    b.init()
    prev = None
    for r in range(6):
        if r == 3:
            b.begin_phase2()
        b.phase2_round() if r >= 3 else b.phase1_round()
        ids, dist, fresh = [t.cpu().numpy() for t in b.graph()]
        # in-round distances come from the Gram form: looser than the reported ones
        srt = np.sort(ids, axis=1)
        assert (srt[:, 1:] != srt[:, :-1]).all() and (ids != np.arange(len(ids))[:, None]).all()
        assert (dist[:, 1:] >= dist[:, :-1]).all()
        ref = _ref_dist(X, np.arange(len(ids)), ids, 0)
        assert np.abs(dist - ref).max() <= 1e-5 * (X.astype(np.float64) ** 2).sum(1).max()
        if prev is not None:
            assert (dist <= prev + 1e-12).all()       # lists only improve
        prev = dist
    b.close()


@pytest.mark.parametrize("metric", ["l2", "ip", "cosine"])
def test_exact_knn_matches_oracle(metric):
    mcode = knn.METRICS[metric]
    # integer-valued rows: fp32 is exact, ids must match bit for bit (ties included)
    X = inputs.make("C2", n=5000, d=24, comps=5)
    rows = inputs.sample_rows(5000, 300)
    ids, dist = knn.exact_knn(torch.from_numpy(X).cuda(), 20, metric, torch.from_numpy(rows))
    oi, od = oracle.brute_force_knn(X, 20, mcode, rows)
    if metric != "cosine":
        assert (ids.cpu().numpy() == oi).all()
        assert (dist.cpu().numpy().astype(np.float64) == od).all()
    else:
        np.testing.assert_allclose(dist.cpu().numpy(), od, rtol=0, atol=2e-6)
    # real-valued rows: a mismatch is allowed only between ids whose fp64 distances agree to 1e-6
    # relative (for cosine: to 5e-7 absolute, a few ulps of the O(1) cosine the fp32 path subtracts from 1)
    X = inputs.make("C1", n=4000)
    ids, dist = knn.exact_knn(torch.from_numpy(X).cuda(), 16, metric)
    oi, od = oracle.brute_force_knn(X, 16, mcode)
    ids = ids.cpu().numpy()
    bad = np.argwhere(ids != oi)
    assert len(bad) < 0.001 * ids.size
    for q, j in bad:
        a = oracle.distance(X, mcode, int(q), int(ids[q, j]))
        tol = 5e-7 if metric == "cosine" else 1e-6 * max(abs(od[q, j]), 1e-3)
        assert abs(a - od[q, j]) <= tol
    _check_properties(X, ids, dist.cpu().numpy().astype(np.float64), mcode)


def test_exact_knn_odd_shapes():
    rng = np.random.default_rng(4)
    X = np.rint(rng.uniform(0, 50, size=(1300, 5))).astype(np.float32)     # d not a multiple of 4, many ties
    ids, dist = knn.exact_knn(torch.from_numpy(X).cuda(), 64, "l2", torch.tensor([0, 1299, 7]))
    oi, od = oracle.brute_force_knn(X, 64, 0, np.array([0, 1299, 7]))
    assert (ids.cpu().numpy() == oi).all() and (dist.cpu().numpy() == od).all()
    with pytest.raises(knn.TagoreError):
        knn.exact_knn(torch.from_numpy(X).cuda(), 8, "l2", torch.tensor([1300]))


def test_degenerate_sizes():
    # k = n - 1: the lists hold every other node from the start and must equal brute force
    X = inputs.make("C2", n=33, d=12, comps=2)
    prm = knn.default_params(32, 4, seed=1)
    ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    oi, od = oracle.brute_force_knn(X, 32)
    assert (ids.cpu().numpy() == oi).all() and (dist.cpu().numpy() == od).all()
    # k = 1, d = 1
    X = inputs.make("C2", n=500, d=1, comps=2)
    prm = knn.default_params(1, 4, seed=1)
    ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    o.run(prm.it1, prm.it2)
    assert (ids.cpu().numpy() == o.graph()[0]).all()
    # no rounds at all: the random lists come back sorted
    prm = knn.default_params(8, 4, seed=9)
    prm.it1 = prm.it2 = 0
    X = inputs.make("C2", n=300, d=16, comps=2)
    ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    o.init()
    assert (ids.cpu().numpy() == o.graph()[0]).all() and st["rounds_phase1"] == 0
    # phase 2 only / phase 1 only
    for it1, it2 in ((0, 3), (3, 0)):
        prm = knn.default_params(8, 4, seed=9)
        prm.it1, prm.it2 = it1, it2
        ids, _, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        o = _oracle_for(X, prm)
        o.run(it1, it2)
        assert (ids.cpu().numpy() == o.graph()[0]).all()


def test_duplicate_points():
    # many identical rows: zero distances and long tie runs
    X = np.repeat(inputs.make("C2", n=60, d=16, comps=2), 20, axis=0)
    prm = knn.default_params(16, 8, seed=2)
    ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    o = _oracle_for(X, prm)
    o.run(prm.it1, prm.it2)
    assert (ids.cpu().numpy() == o.graph()[0]).all()
    _check_properties(X, ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64))


@pytest.mark.parametrize("metric", ["l2", "ip", "cosine"])
def test_rows_without_a_defined_distance_are_counted_and_leave_valid_lists(metric):
    """Zero rows under the cosine distance (0 / 0) and rows with infinite or undefined values have no
    defined distances.  The build counts them (stats: undefined_rows) instead of refusing them; the lists
    are then unspecified, but no distance ever becomes an index, so every list still holds ids in range,
    never its own node and no id twice, and the call succeeds."""
    n, k = 3000, 16
    X = inputs.make("C4", n=n, d=24, comps=6)
    prm = knn.default_params(k, 6, metric=metric, seed=4)
    _, _, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    assert st["undefined_rows"] == 0
    X[5::97] = 0.0                                   # no direction
    X[11::211, 3] = np.inf
    X[17::223, 7] = -np.inf
    X[23::227, 0] = np.nan
    X[29::229, 1] = 3e19                             # a finite value whose square is not
    with np.errstate(over="ignore", invalid="ignore"):
        bad = ~np.isfinite((X.astype(np.float64) ** 2).sum(axis=1).astype(np.float32))
    if metric == "cosine":
        bad |= (X == 0).all(axis=1)
    ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
    assert st["undefined_rows"] == bad.sum() > 0
    ids = ids.cpu().numpy()
    assert ids.shape == (n, k) and (ids >= 0).all() and (ids < n).all()
    assert (ids != np.arange(n)[:, None]).all()
    s = np.sort(ids, axis=1)
    assert (s[:, 1:] != s[:, :-1]).all()


def test_f16_join_counts_rows_beyond_the_fp16_range():
    """join_f16 = 1 rounds every row to fp16 whatever its values: a row with a finite value beyond +-65504 has
    no fp16 copy to rank on.  Such rows are counted once each (stats: undefined_rows); every list stays
    well-formed and holds exact distances (arrivals are measured again in fp32).  With join_f16 = 2 the same data
    take the fp32 join, and nothing is counted."""
    n, k = 2500, 16
    X = inputs.make("C1", n=n, d=40)
    rows = np.array([7, 300, 301, 2499])
    X[rows, 3] = 7.0e4
    X[300, 21] = -1.0e5           # twice in one row, in two pieces of the row: still one row
    X[301, 39] = 9.0e4
    Xg = torch.from_numpy(X).cuda()
    prm = knn.default_params(k, 6, seed=3, join_f16=1)
    ids, dist, st = knn.knn_build_ex(Xg, prm)
    assert st["undefined_rows"] == len(rows)
    _check_properties(X, ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64))
    prm2 = knn.default_params(k, 6, seed=3, join_f16=2)
    ids2, _, st2 = knn.knn_build_ex(Xg, prm2)
    ids0, _, st0 = knn.knn_build_ex(Xg, knn.default_params(k, 6, seed=3))
    assert st2["undefined_rows"] == 0 and st0["undefined_rows"] == 0
    assert (ids2 == ids0).all()


def test_set_graph_round_trip_and_stream():
    X = inputs.make("C2", n=800, d=20, comps=2)
    prm = knn.default_params(12, 4, seed=6)
    o = _oracle_for(X, prm)
    o.init()
    o.phase1_round()
    oi, od, of = o.graph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                       # all work goes to the caller's stream
        b = knn.Builder(torch.from_numpy(X).cuda(), prm)
        b.set_graph(torch.from_numpy(oi), torch.from_numpy(od), torch.from_numpy(of))
        assert _same(b.graph(), (oi, od, of))
        b.begin_phase2(); o.begin_phase2()
        assert b.phase2_round() == o.phase2_round()
        assert _same(b.graph(), o.graph())
        b.close()


# ---- the local join on f16 matrix instructions (join_f16 = 1) ---------------------------------------------

def _f16(X):
    """Round to nearest even to f16, by torch's conversion (independent of the library's)."""
    return torch.from_numpy(np.ascontiguousarray(X)).to(torch.float16).to(torch.float64).numpy()


@pytest.mark.parametrize("d", [4, 32, 50, 64, 100, 128, 200, 960])
def test_f16_join_distance_tile(d):
    """Both join cores (register-resident for small blocks of short rows, LDS tiles otherwise) with join_f16 = 1:
    fp32 norms of the vectors as given, inner products of the vectors rounded to f16 (a truncating conversion,
    or a wrong operand layout of the wider matrix instruction, would be far outside the tolerance)."""
    n = 600
    rng = np.random.default_rng(100 + d)
    X = rng.standard_normal((n, d)).astype(np.float32)
    b = knn.Builder(torch.from_numpy(X).cuda(), knn.default_params(16, 4, join_f16=1))
    shapes = [(32, 32), (1, 1), (17, 30), (64, 0), (5, 0), (16, 16), (2, 0), (1, 63), (40, 24), (33, 15), (64, 64), (48, 49),
              (33, 95), (1, 127)]
    blk = np.zeros((len(shapes), 128), dtype=np.int32)
    sizes = np.zeros((len(shapes), 2), dtype=np.int32)
    for i, (a, o) in enumerate(shapes):
        blk[i, :a + o] = rng.choice(n, size=a + o, replace=False)
        sizes[i] = (a, o)
    out = b.join_distances(torch.from_numpy(blk), torch.from_numpy(sizes)).cpu().numpy()
    Xr = _f16(X)
    nrm = (X.astype(np.float64) ** 2).sum(1)
    tol = 4e-6 * nrm.max()
    worst_vs_unrounded = 0.0
    for i, (a, o) in enumerate(shapes):
        idx = blk[i, :a + o]
        ref = nrm[idx][:, None] + nrm[idx][None, :] - 2.0 * Xr[idx] @ Xr[idx].T
        exact = nrm[idx][:, None] + nrm[idx][None, :] - 2.0 * X[idx].astype(np.float64) @ X[idx].astype(np.float64).T
        used = np.zeros((a, a + o), dtype=bool)
        for r in range(a):
            used[r, r + 1:] = True
        got = out[i][:a, :a + o]
        assert np.abs(got[used] - ref[:a][used]).max() <= tol
        if used.any():
            worst_vs_unrounded = max(worst_vs_unrounded, np.abs(got[used] - exact[:a][used]).max())
    assert worst_vs_unrounded > tol, "the rounded copy was not used"
    b.close()


@pytest.mark.parametrize("n,d,k,kw", [(3000, 64, 32, dict(C=64)), (1400, 128, 32, dict(C=256)), (1200, 30, 10, dict(C=32)),
                                      (1500, 100, 24, dict(C=128)), (900, 256, 32, dict(C=64)), (800, 300, 48, dict(C=128)),
                                      (1000, 64, 16, dict(C=32, parts=2))])
def test_f16_join_is_exact_on_representable_data(n, d, k, kw):
    """Byte-valued features (and eighths of them) are f16 numbers: the rounded copy is exact, products and sums are
    exact in fp32, so the graph must equal the oracle's bit for bit."""
    Xi = inputs.make("C2", n=n, d=d, comps=max(2, n // 500))
    if d > 128:
        Xi = np.floor(Xi / 4)                 # squared norms stay below 2^23
    for X in (Xi, np.floor(Xi / 8) / 8):
        X = np.ascontiguousarray(X, dtype=np.float32)
        assert (_f16(X) == X).all()
        prm = knn.default_params(k, 8, seed=7, join_f16=1, **kw)
        ids, dist, st = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        o = _oracle_for(X, prm)
        o.run(prm.it1, prm.it2)
        oi, od, _ = o.graph()
        assert (ids.cpu().numpy() == oi).all()
        assert (dist.cpu().numpy().astype(np.float64) == od).all()


@pytest.mark.parametrize("cfg,metric", [("C1", "l2"), ("C4", "cosine"), ("C4", "ip"), ("C3", "l2")])
def test_f16_join_statistical_parity_on_real_valued_data(cfg, metric):
    """Real-valued data: the join ranks on rounded vectors, so parity is what it is for the fp32 join: recall within
    0.005 of the oracle's (mean of 3 seeds), reported distances exact to 1e-4 of fp64, lists well-formed."""
    sizes = {"C1": dict(n=6000), "C4": dict(n=5000, comps=10), "C3": dict(n=3000, d=200, comps=6)}[cfg]
    X = inputs.make(cfg, **sizes)
    k = 16
    mcode = knn.METRICS[metric]
    truth, _ = oracle.brute_force_knn(X, k, mcode)
    gaps = []
    for seed in (1, 2, 3):
        prm = knn.default_params(k, 6, metric=metric, seed=seed, C=32, join_f16=1, it1=3, it2=3)
        ids, dist, _ = knn.knn_build_ex(torch.from_numpy(X).cuda(), prm)
        ids, dist = ids.cpu().numpy(), dist.cpu().numpy().astype(np.float64)
        _check_properties(X, ids, dist, mcode)
        o = _oracle_for(X, knn.default_params(k, 6, metric=metric, seed=seed, C=32, it1=3, it2=3), mcode)
        o.run(prm.it1, prm.it2)
        gaps.append(oracle.recall(ids, truth) - oracle.recall(o.graph()[0], truth))
    assert np.mean(gaps) >= -RECALL_TOL, gaps


@pytest.mark.parametrize("n,d,k,kw", [(2000, 128, 32, dict(C=128)), (1200, 200, 16, dict(C=64)), (1500, 48, 24, dict(C=64, parts=1))])
def test_f16_join_only_where_exact(n, d, k, kw):
    """join_f16 = 2 narrows only when every value is an f16 number: on such data the graph equals the oracle's, on
    real-valued data it equals the fp32 join's, bit for bit either way."""
    Xi = inputs.make("C2", n=n, d=d, comps=4)
    if d > 128:
        Xi = np.floor(Xi / 4)
    prm = knn.default_params(k, 6, seed=3, join_f16=2, **kw)
    ids, dist, _ = knn.knn_build_ex(torch.from_numpy(Xi).cuda(), prm)
    o = _oracle_for(Xi, prm)
    o.run(prm.it1, prm.it2)
    oi, od, _ = o.graph()
    assert (ids.cpu().numpy() == oi).all() and (dist.cpu().numpy().astype(np.float64) == od).all()
    Xr = inputs.make("C1", n=n, d=d)
    Xr[n // 2, d // 2] = np.float32(1.0) + np.float32(2.0) ** -20          # one value that is no f16 number is enough
    a_ids, a_dist, _ = knn.knn_build_ex(torch.from_numpy(Xr).cuda(), prm)
    b_ids, b_dist, _ = knn.knn_build_ex(torch.from_numpy(Xr).cuda(), knn.default_params(k, 6, seed=3, join_f16=0, **kw))
    assert bool((a_ids == b_ids).all()) and bool((a_dist == b_dist).all())
    forced, _, _ = knn.knn_build_ex(torch.from_numpy(Xr).cuda(), knn.default_params(k, 6, seed=3, join_f16=1, **kw))
    assert not bool((forced == b_ids).all()), "rounding real-valued rows should change some decisions"


def test_list_operations_need_lists_and_valid_ids():
    X = torch.zeros((200, 8), device="cuda")
    b = knn.Builder(X, knn.default_params(4, 2))
    for call in (b.phase1_round, b.begin_phase2, b.phase2_round, b.finalize, b.graph, b.sample_blocks):
        with pytest.raises(knn.TagoreError):
            call()
    ids = torch.zeros((200, 4), dtype=torch.int32, device="cuda")
    ids[17, 2] = 200
    dist, fresh = torch.zeros((200, 4), device="cuda"), torch.zeros((200, 4), dtype=torch.uint8, device="cuda")
    # (the binding has a check of its own; this is the library's, through the C boundary)
    assert knn.lib().tg_knn_import(b._h, ids.data_ptr(), dist.data_ptr(), fresh.data_ptr()) == -1
    assert b"out of range" in knn.lib().tg_last_error()
    b.init()
    b.phase1_round()
    b.close()


def test_exact_knn_refuses_rows_outside_the_data():
    X = torch.from_numpy(inputs.make("C1", n=500)).cuda()
    for bad in (500, -7, 10**9):
        with pytest.raises(knn.TagoreError):
            knn.exact_knn(X, 5, "l2", torch.tensor([3, bad, 499], dtype=torch.int64))
