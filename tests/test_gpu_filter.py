"""Distance-based pruning (NSG / Vamana rule of section 3.2 in the Collect-Filter-Store procedure of
section 5.1) on the GPU against the oracle.

On integer-valued data whose squared norms stay below 2^23 every fp32 value either side forms is
exact, so the rows must agree bit for bit.  On real-valued data the GPU's distances carry fp32
rounding (about (d + 8) 2^-24 of the squared norms involved): a row may differ from the oracle's only
if the oracle says that one of its decisions was that close to flipping, and few rows may."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def _integer_points(n, d, comps=12, shrink=1):
    X = inputs.make("C2", n=n, d=d, comps=comps)
    return np.floor(X / shrink).astype(np.float32)


def _exact(X, ids, d_out, alpha, hops, cand_size):
    want, want_deg, _ = oracle.filter_dist(X, ids, hops, cand_size, alpha, d_out)
    out, deg = knn.prune_dist(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), d_out, alpha=alpha, hops=hops,
                              cand_size=cand_size, want_degrees=True)
    out, deg = out.cpu().numpy(), deg.cpu().numpy()
    bad = np.nonzero((out != want).any(axis=1))[0]
    assert bad.size == 0, (bad[:5], out[bad[:2]], want[bad[:2]])
    assert (deg == want_deg).all()
    return want, want_deg


@pytest.mark.parametrize("n,d,k,d_out,alpha,cand_size", [
    (3000, 128, 32, 16, 1.0, 64),       # the headline shape: two row groups, one chunk of columns
    (3000, 128, 32, 32, 1.2, 64),
    (2000, 128, 64, 32, 1.0, 64),       # four row groups
    (2000, 128, 48, 48, 1.5, 40),       # cand_size cuts the candidates
    (1500, 64, 24, 8, 1.1, 64),         # half a chunk of columns
    (1200, 96, 32, 16, 1.0, 64),
    (900, 100, 17, 17, 1.3, 64),
    (700, 30, 9, 4, 1.0, 64),           # rows that are not 16-byte aligned
    (600, 3, 5, 5, 2.0, 64),
    (300, 1, 1, 1, 1.0, 1),
])
def test_one_hop_bit_exact_on_integer_data(n, d, k, d_out, alpha, cand_size):
    X = _integer_points(n, d)
    ids, _ = oracle.brute_force_knn(X, k)
    _exact(X, ids, d_out, alpha, 1, cand_size)


@pytest.mark.parametrize("n,d,k,d_out,alpha,cand_size", [
    (2500, 128, 32, 32, 1.0, 64),
    (2000, 128, 16, 24, 1.2, 64),
    (1500, 64, 20, 20, 1.0, 33),
    (800, 30, 7, 12, 1.4, 64),
    (500, 8, 3, 6, 1.0, 5),
    (1200, 128, 64, 32, 1.0, 64),       # rows of more than 32 ids: the instance with the larger id set
    (900, 48, 40, 24, 1.3, 50),
    (700, 20, 33, 64, 1.1, 64),
])
def test_two_hops_bit_exact_on_integer_data(n, d, k, d_out, alpha, cand_size):
    X = _integer_points(n, d)
    ids, _ = oracle.brute_force_knn(X, k)
    _exact(X, ids, d_out, alpha, 2, cand_size)


@pytest.mark.parametrize("d,hops", [(960, 1), (300, 2), (260, 1)])
def test_several_chunks_of_columns(d, hops):
    X = _integer_points(1000, d, shrink=8)        # values 0..31: squared norms below 2^20
    ids, _ = oracle.brute_force_knn(X, 32 if hops == 1 else 12)
    _exact(X, ids, 16, 1.0, hops, 64)
    _exact(X, ids, 16, 1.25, hops, 64)


def test_unaligned_base_pointer():
    X = _integer_points(1200, 128)
    ids, _ = oracle.brute_force_knn(X, 32)
    buf = torch.empty(X.size + 1, dtype=torch.float32, device="cuda")
    Xg = buf[1:].view(X.shape)                     # 4 bytes past a 16-byte boundary
    Xg.copy_(torch.from_numpy(X))
    assert Xg.data_ptr() % 16 == 4
    want, _, _ = oracle.filter_dist(X, ids, 1, 64, 1.0, 16)
    out = knn.prune_dist(Xg, torch.from_numpy(ids).cuda(), 16)
    assert (out.cpu().numpy() == want).all()


def test_graph_from_the_builder():
    X = inputs.make("C2", n=20000, d=128, comps=20)
    Xg = torch.from_numpy(X).cuda()
    ids, _ = knn.knn_build(Xg, 32, "l2", iters=8, seed=1)
    ids = ids.cpu().numpy()
    want, deg = _exact(X, ids, 16, 1.0, 1, 64)
    # alpha = 1 thins the rows out; a larger alpha keeps more (section 3.2: Vamana relaxes NSG's rule)
    _, deg12 = _exact(X, ids, 16, 1.2, 1, 64)
    assert deg.mean() < deg12.mean() <= 16 and deg.min() >= 1
    assert (want[:, 0] == ids[:, 0]).all()          # the nearest neighbour is always inserted
    _exact(X[:6000], ids[:6000] % 6000, 24, 1.1, 2, 64)


def test_padding_duplicates_self_and_small_candidate_sets():
    rng = np.random.default_rng(5)
    n, k, d = 800, 16, 40
    X = _integer_points(n, d)
    X[1::7] = X[0::7][: len(X[1::7])]                                       # twins
    ids = np.stack([rng.permutation(n)[:k] for _ in range(n)]).astype(np.int32)
    ids[rng.integers(0, n, 300), rng.integers(0, k, 300)] = -1            # padding
    ids[rng.integers(0, n, 100), rng.integers(0, k, 100)] = n + 7         # ids without a row
    rows = rng.integers(0, n, 100)
    ids[rows, 5] = ids[rows, 2]                                            # an id listed twice
    ids[:50, 3] = np.arange(50)                                            # a node in its own row
    ids[60:70] = -1                                                        # rows without any candidate
    for hops in (1, 2):
        for alpha in (1.0, 1.3, 1000.0):
            want, deg = _exact(X, ids, 20, alpha, hops, 64)
            assert (want[60:70] == -1).all() and (deg[60:70] == 0).all()


def test_wide_rows_with_padding_and_repeats_over_two_hops():
    # rows of 40 and of 64 ids (the two-hop instance with the larger id set), with padding, ids without a row,
    # repeats, self ids, empty rows and twins among the points
    rng = np.random.default_rng(6)
    n, d = 600, 24
    X = _integer_points(n, d)
    X[1::5] = X[0::5][: len(X[1::5])]
    for k in (40, 64):
        ids = rng.integers(0, n, size=(n, k)).astype(np.int32)
        noise = rng.random((n, k))
        ids[noise < 0.1] = -1
        ids[(noise >= 0.1) & (noise < 0.13)] = n + 3
        ids[:40, 7] = np.arange(40)
        ids[100:110] = -1
        for alpha, d_out, cand_size in ((1.0, 32, 64), (1.4, 64, 47)):
            want, deg = _exact(X, ids, d_out, alpha, 2, cand_size)
            assert (deg[100:110] == 0).all()
        want, want_deg, _ = oracle.filter_angle(X, ids, 2, 64, 60.0, 24)
        out = knn.prune_angle(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), 24, gamma_deg=60.0, hops=2)
        assert (out.cpu().numpy() == want).all()
        want, want_deg, _ = oracle.filter_dpg(X, ids, 2, 64, 24)
        out = knn.prune_dispersion(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), 24, hops=2)
        assert (out.cpu().numpy() == want).all()


@pytest.mark.parametrize("config,n,d,k,hops", [("C1", 4000, 32, 16, 1), ("C1", 3000, 32, 16, 2), ("C4", 3000, 96, 32, 1),
                                               ("C3", 1500, 960, 32, 1)])
def test_real_valued_data_differs_only_where_a_decision_was_a_near_tie(config, n, d, k, hops):
    X = inputs.make(config, n=n, d=d, comps=10)
    ids, _ = oracle.brute_force_knn(X, k)
    for alpha in (1.0, 1.2):
        want, want_deg, margin = oracle.filter_dist(X, ids, hops, 64, alpha, 16)
        out = knn.prune_dist(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(), 16, alpha=alpha, hops=hops).cpu().numpy()
        differ = (out != want).any(axis=1)
        tol = 4.0 * (d + 8) * 2.0 ** -24 * max(1.0, alpha * alpha)
        assert (margin[differ] < tol).all(), (np.nonzero(differ)[0][:5], margin[differ][:5], tol)
        assert differ.mean() < 0.02, differ.mean()


def test_bad_arguments():
    X = torch.zeros((100, 8), device="cuda")
    ids = torch.zeros((100, 40), dtype=torch.int32, device="cuda")
    for kw in (dict(d_out=0), dict(d_out=65), dict(d_out=4, alpha=0.9), dict(d_out=4, hops=3), dict(d_out=4, cand_size=0),
               dict(d_out=4, cand_size=65)):
        with pytest.raises(knn.TagoreError):
            knn.prune_dist(X, ids, **kw)
