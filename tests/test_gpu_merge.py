"""Merge of local indexes into the global lists (section 6.1) on the GPU against the oracle: ids are
integer work and distances are copied, so everything must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def _merge_both(n, k, shards):
    """shards: list of (l_ids, l_dist, l2g) numpy arrays.  Returns the oracle's lists after checking the GPU's."""
    w_ids = np.full((n, k), -1, dtype=np.int32)
    w_dist = np.full((n, k), np.inf, dtype=np.float32)
    g_ids, g_dist = knn.lists_clear(n, k)
    assert (g_ids.cpu().numpy() == w_ids).all() and (g_dist.cpu().numpy() == w_dist).all()
    for l_ids, l_dist, l2g in shards:
        oracle.merge_local(w_ids, w_dist, l_ids, l_dist, l2g)
        knn.merge_local(g_ids, g_dist, torch.from_numpy(l_ids).cuda(), torch.from_numpy(l_dist).cuda(),
                        torch.from_numpy(l2g).cuda())
        assert (g_ids.cpu().numpy() == w_ids).all()
        assert (g_dist.cpu().numpy() == w_dist).all()
    return w_ids, w_dist


@pytest.mark.parametrize("n,d,k,k_local,size,count", [(3000, 16, 32, 32, 1200, 6), (2000, 8, 16, 64, 900, 5),
                                                     (1500, 8, 64, 24, 700, 7), (500, 4, 5, 3, 100, 9), (300, 2, 1, 1, 50, 4)])
def test_exact_local_indexes(n, d, k, k_local, size, count):
    rng = np.random.default_rng(n + k)
    X = np.floor(inputs.make("C2", n=n, d=d, comps=8) / 4).astype(np.float32)      # ties and twins on purpose
    shards = []
    for _ in range(count):
        members = np.sort(rng.permutation(n)[:size]).astype(np.int32)
        rng.shuffle(members)                                                      # any order of the cluster's rows
        ids, dist = oracle.brute_force_knn(X[members], k_local)
        shards.append((ids, dist.astype(np.float32), members))
    _merge_both(n, k, shards)


def test_padding_self_repeats_and_ids_without_a_node():
    rng = np.random.default_rng(11)
    n, k, kl, nl = 400, 12, 20, 150
    shards = []
    for s in range(4):
        l2g = rng.permutation(n)[:nl].astype(np.int32)
        l_ids = rng.integers(0, nl, size=(nl, kl)).astype(np.int32)               # repeats inside rows, self ids
        l_dist = rng.integers(0, 40, size=(nl, kl)).astype(np.float32)            # the same id with other distances
        l_ids[rng.integers(0, nl, 200), rng.integers(0, kl, 200)] = -1
        l_ids[rng.integers(0, nl, 50), rng.integers(0, kl, 50)] = nl + 3
        shards.append((l_ids, l_dist, l2g))
    _merge_both(n, k, shards)


def test_a_local_node_without_a_global_row_is_skipped():
    n, k = 50, 4
    g_ids, g_dist = knn.lists_clear(n, k)
    l2g = torch.tensor([3, 70, 5, -2], dtype=torch.int32, device="cuda")
    l_ids = torch.tensor([[1, 2, 3], [0, 2, 3], [0, 1, 3], [0, 1, 2]], dtype=torch.int32, device="cuda")
    l_dist = torch.tensor([[1, 2, 3], [1, 4, 5], [2, 4, 6], [3, 5, 6]], dtype=torch.float32, device="cuda")
    knn.merge_local(g_ids, g_dist, l_ids, l_dist, l2g)
    got = g_ids.cpu().numpy()
    assert list(got[3]) == [5, -1, -1, -1] and list(got[5]) == [3, -1, -1, -1]     # neighbours 70 and -2 are no nodes
    assert (np.delete(got, [3, 5], axis=0) == -1).all()
    wide_ids, wide_dist = knn.lists_clear(10, 65)
    with pytest.raises(knn.TagoreError):
        knn.merge_local(wide_ids, wide_dist, l_ids, l_dist, l2g)                   # k > 64
    with pytest.raises(knn.TagoreError):
        knn.lists_clear(10, 0)


def test_sharded_build_then_merge():
    # clusters as in section 6.1: every point goes to its 2 closest of 6 centres; each cluster is built on its own
    # and merged.  Parity: the merged lists equal the oracle's merge of the same local indexes.  Quality: recall of
    # the merged graph is close to that of one build over all points.
    n, d, k = 40000, 64, 32
    X = inputs.make("C2", n=n, d=d, comps=30)
    Xg = torch.from_numpy(X).cuda()
    rng = np.random.default_rng(2)
    centres = Xg[torch.from_numpy(rng.permutation(n)[:6]).cuda()]
    near = torch.cdist(Xg, centres).topk(2, dim=1, largest=False).indices
    shards = []
    for c in range(6):
        members = torch.nonzero((near == c).any(dim=1)).flatten().to(torch.int32)
        if members.numel() <= k:
            continue
        ids, dist = knn.knn_build(Xg[members.long()].contiguous(), k, "l2", iters=10, seed=1)
        shards.append((ids.cpu().numpy(), dist.cpu().numpy(), members.cpu().numpy()))
    assert sum(s[2].size for s in shards) == 2 * n
    w_ids, w_dist = _merge_both(n, k, shards)
    rows = inputs.sample_rows(n, 1000, seed=4)
    truth, _ = oracle.brute_force_knn(X, k, 0, rows)
    whole, _ = knn.knn_build(Xg, k, "l2", iters=10, seed=1)
    rec_merged = oracle.recall(w_ids[rows], truth)
    rec_whole = oracle.recall(whole.cpu().numpy()[rows], truth)
    assert rec_merged > rec_whole - 0.03 and rec_merged > 0.9, (rec_merged, rec_whole)
