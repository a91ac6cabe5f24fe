"""Rank-based pruning (sections 3.2 and 5.2) on the GPU against the oracle: integer work, so bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def _check(ids, d_out):
    want_out, want_cnt = oracle.prune_rank(ids, d_out)
    out, cnt = knn.prune_rank(torch.from_numpy(ids).cuda(), d_out, want_counts=True)
    assert (cnt.cpu().numpy() == want_cnt).all()
    assert (out.cpu().numpy() == want_out).all()
    assert (knn.prune_rank(torch.from_numpy(ids).cuda(), d_out).cpu().numpy() == want_out).all()


@pytest.mark.parametrize("n,d,k,d_out", [(3000, 8, 32, 16), (2000, 4, 64, 32), (1500, 16, 24, 24), (700, 3, 5, 2),
                                         (260, 2, 1, 1), (1000, 6, 33, 7)])
def test_exact_graphs(n, d, k, d_out):
    X = inputs.make("C1", n=n, d=d)
    ids, _ = oracle.brute_force_knn(X, k)
    _check(ids, d_out)


def test_graph_from_the_builder_and_recall_of_what_is_kept():
    X = inputs.make("C2", n=20000, d=64, comps=20)
    ids, _ = knn.knn_build(torch.from_numpy(X).cuda(), 32, "l2", iters=8, seed=1)
    ids = ids.cpu().numpy()
    _check(ids, 16)
    out, cnt = oracle.prune_rank(ids, 16)
    # every kept neighbour is one of the row's neighbours, none twice; close neighbours are rarely detoured
    assert all(len(set(out[v])) == 16 and set(out[v]) <= set(ids[v]) for v in range(0, 20000, 97))
    assert cnt[:, 1:].mean() > 0.5 and (out[:, 0] == ids[:, 0]).all()


def test_padding_duplicates_and_bad_arguments():
    rng = np.random.default_rng(5)
    n, k = 800, 16
    ids = np.stack([rng.permutation(n)[:k] for _ in range(n)]).astype(np.int32)
    ids[rng.integers(0, n, 300), rng.integers(0, k, 300)] = -1            # padding
    ids[rng.integers(0, n, 100), rng.integers(0, k, 100)] = n + 7         # ids without a row
    rows = rng.integers(0, n, 100)
    ids[rows, 5] = ids[rows, 2]                                            # an id listed twice
    ids[:50, 3] = np.arange(50)                                            # a node in its own row
    _check(ids, 9)
    # few nodes: every row shares most of its ids with every other, so repeats, own ids, padding and ids
    # without a row all sit where detours are counted
    for n2, k2, seed in ((40, 16, 1), (24, 20, 2), (70, 33, 3), (100, 64, 4)):
        r2 = np.random.default_rng(seed)
        dense = r2.integers(0, n2, (n2, k2)).astype(np.int32)              # with repeats and own ids
        dense[r2.random((n2, k2)) < 0.05] = -1
        dense[r2.random((n2, k2)) < 0.05] = n2 + 7
        _check(dense, max(1, k2 // 2))
        _check(dense, k2)
    t = torch.from_numpy(ids).cuda()
    for bad in (0, k + 1):
        with pytest.raises(knn.TagoreError):
            knn.prune_rank(t, bad)
