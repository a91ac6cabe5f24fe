"""Angle-based pruning (the NSSG rule of section 3.2 in the Collect-Filter-Store procedure of section
5.1) on the GPU against the oracle.

On integer-valued data whose squared norms stay below 2^23 the squared lengths a, b, c and t = a + b - c
are exact in fp32 on both sides, and t * t, a * b and their product with 4 cos^2(gamma) are single
roundings of the same operands, so the rows must agree bit for bit.  On real-valued data a row may
differ only where the oracle reports a decision within fp32 rounding of its threshold."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def _integer_points(n, d, comps=12, shrink=1):
    X = inputs.make("C2", n=n, d=d, comps=comps)
    return np.floor(X / shrink).astype(np.float32)


def _exact(X, ids, d_out, gamma, hops, cand_size):
    want, want_deg, _ = oracle.filter_angle(X, ids, hops, cand_size, gamma, d_out)
    out, deg = knn.prune_angle(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), d_out, gamma_deg=gamma, hops=hops,
                               cand_size=cand_size, want_degrees=True)
    out, deg = out.cpu().numpy(), deg.cpu().numpy()
    bad = np.nonzero((out != want).any(axis=1))[0]
    assert bad.size == 0, (bad[:5], out[bad[:2]], want[bad[:2]])
    assert (deg == want_deg).all()
    return want, want_deg


@pytest.mark.parametrize("n,d,k,d_out,gamma,cand_size", [
    (3000, 128, 32, 16, 60.0, 64),      # the headline shape: two row groups, one chunk of columns
    (3000, 128, 32, 32, 45.0, 64),
    (2000, 128, 64, 32, 60.0, 64),      # four row groups
    (2000, 128, 48, 48, 30.0, 40),      # cand_size cuts the candidates
    (1500, 64, 24, 8, 75.0, 64),
    (1200, 96, 32, 16, 90.0, 64),       # cos = 0: only obtuse angles pass
    (900, 100, 17, 17, 52.5, 64),
    (700, 30, 9, 4, 60.0, 64),          # rows that are not 16-byte aligned
    (600, 3, 5, 5, 20.0, 64),
    (300, 1, 1, 1, 60.0, 1),
])
def test_one_hop_bit_exact_on_integer_data(n, d, k, d_out, gamma, cand_size):
    X = _integer_points(n, d)
    ids, _ = oracle.brute_force_knn(X, k)
    _exact(X, ids, d_out, gamma, 1, cand_size)


@pytest.mark.parametrize("n,d,k,d_out,gamma,cand_size", [
    (2500, 128, 32, 32, 60.0, 64),
    (2000, 128, 16, 24, 40.0, 64),
    (1500, 64, 20, 20, 90.0, 33),
    (800, 30, 7, 12, 70.0, 64),
    (500, 8, 3, 6, 60.0, 5),
    (1200, 128, 64, 32, 60.0, 64),      # rows of more than 32 ids: the instance with the larger id set
    (900, 48, 40, 24, 45.0, 50),
])
def test_two_hops_bit_exact_on_integer_data(n, d, k, d_out, gamma, cand_size):
    X = _integer_points(n, d)
    ids, _ = oracle.brute_force_knn(X, k)
    _exact(X, ids, d_out, gamma, 2, cand_size)


@pytest.mark.parametrize("d,hops", [(960, 1), (300, 2)])
def test_several_chunks_of_columns(d, hops):
    X = _integer_points(1000, d, shrink=8)        # values 0..31: squared norms below 2^20
    ids, _ = oracle.brute_force_knn(X, 32 if hops == 1 else 12)
    _exact(X, ids, 16, 60.0, hops, 64)


def test_graph_from_the_builder():
    X = inputs.make("C2", n=20000, d=128, comps=20)
    Xg = torch.from_numpy(X).cuda()
    ids, _ = knn.knn_build(Xg, 32, "l2", iters=8, seed=1)
    ids = ids.cpu().numpy()
    want, deg60 = _exact(X, ids, 16, 60.0, 1, 64)
    _, deg40 = _exact(X, ids, 16, 40.0, 1, 64)
    _, deg90 = _exact(X, ids, 16, 90.0, 1, 64)
    assert 1 <= deg90.mean() < deg60.mean() < deg40.mean() <= 16 and deg90.min() >= 1    # a wider cone drops more
    assert (want[:, 0] == ids[:, 0]).all()          # the nearest neighbour is always inserted
    _exact(X[:6000], ids[:6000] % 6000, 24, 60.0, 2, 64)


def test_padding_duplicates_self_and_small_candidate_sets():
    rng = np.random.default_rng(5)
    n, k, d = 800, 16, 40
    X = _integer_points(n, d)
    X[1::7] = X[0::7][: len(X[1::7])]                                       # twins: also candidates at p's own position
    ids = np.stack([rng.permutation(n)[:k] for _ in range(n)]).astype(np.int32)
    ids[rng.integers(0, n, 300), rng.integers(0, k, 300)] = -1
    ids[rng.integers(0, n, 100), rng.integers(0, k, 100)] = n + 7
    rows = rng.integers(0, n, 100)
    ids[rows, 5] = ids[rows, 2]
    ids[:50, 3] = np.arange(50)
    ids[0:700:7, 0] = np.arange(1, 701, 7)                                  # every such p lists its twin
    ids[60:70] = -1
    for hops in (1, 2):
        for gamma in (10.0, 60.0, 90.0):
            want, deg = _exact(X, ids, 20, gamma, hops, 64)
            assert (want[60:70] == -1).all() and (deg[60:70] == 0).all()


@pytest.mark.parametrize("config,n,d,k,hops", [("C1", 4000, 32, 16, 1), ("C1", 3000, 32, 16, 2), ("C4", 3000, 96, 32, 1),
                                               ("C3", 1500, 960, 32, 1)])
def test_real_valued_data_differs_only_where_a_decision_was_a_near_tie(config, n, d, k, hops):
    X = inputs.make(config, n=n, d=d, comps=10)
    ids, _ = oracle.brute_force_knn(X, k)
    for gamma in (60.0, 40.0):
        want, want_deg, margin = oracle.filter_angle(X, ids, hops, 64, gamma, 16)
        out = knn.prune_angle(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), 16, gamma_deg=gamma, hops=hops).cpu().numpy()
        differ = (out != want).any(axis=1)
        # t = a + b - c carries the rounding of three squared lengths, each about (d + 8) 2^-24 of the norms
        tol = 8.0 * (d + 8) * 2.0 ** -24
        assert (margin[differ] < tol).all(), (np.nonzero(differ)[0][:5], margin[differ][:5], tol)
        assert differ.mean() < 0.02, differ.mean()


def test_bad_arguments():
    X = torch.zeros((100, 8), device="cuda")
    ids = torch.zeros((100, 40), dtype=torch.int32, device="cuda")
    for kw in (dict(d_out=0), dict(d_out=65), dict(d_out=4, gamma_deg=0.0), dict(d_out=4, gamma_deg=91.0),
               dict(d_out=4, gamma_deg=float("nan")), dict(d_out=4, hops=3), dict(d_out=4, cand_size=0),
               dict(d_out=4, cand_size=65)):
        with pytest.raises(knn.TagoreError):
            knn.prune_angle(X, ids, **kw)
