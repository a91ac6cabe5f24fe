"""The allocation-free exact k-NN (tg_exact_knn_static) against tg_exact_knn, through the C-ABI."""
import numpy as np
import pytest
import torch

from paper_2508_08744_amd import inputs, knn

pytestmark = pytest.mark.gpu


def _same(a, b):
    return torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_static_scratch_matches_the_allocating_entry_point_twice_in_a_row():
    dev = "cuda:0"
    # first call: cosine (norms in the scratch), several slices, a ragged tail of queries
    X1 = torch.from_numpy(inputs.make("C4", n=30_011)).to(dev)
    rows1 = torch.from_numpy(inputs.sample_rows(30_011, 1_003)).to(dev)
    want1 = knn.exact_knn(X1, 32, "cosine", rows1)
    got1 = knn.exact_knn_static(X1, 32, "cosine", rows1)
    torch.cuda.synchronize()
    assert _same(got1, want1)
    # second call right behind it, smaller, another metric: the scratch still holds the first call's words
    X2 = torch.from_numpy(inputs.make("C2", n=5_000, d=64, comps=20)).to(dev)
    rows2 = torch.arange(0, 5_000, 7, dtype=torch.int64, device=dev)
    want2 = knn.exact_knn(X2, 10, "l2", rows2)
    got2 = knn.exact_knn_static(X2, 10, "l2", rows2)
    torch.cuda.synchronize()
    assert _same(got2, want2)
    # all rows as queries (no row list), inner product
    want3 = knn.exact_knn(X2, 16, "ip")
    got3 = knn.exact_knn_static(X2, 16, "ip")
    torch.cuda.synchronize()
    assert _same(got3, want3)
    # and the first problem again: nothing of the smaller calls is left in the way
    got4 = knn.exact_knn_static(X1, 32, "cosine", rows1)
    torch.cuda.synchronize()
    assert _same(got4, want1)


def test_static_scratch_refuses_what_does_not_fit_and_what_would_need_a_copy():
    dev = "cuda:0"
    X = torch.from_numpy(inputs.make("C2", n=4_000, d=64, comps=8)).to(dev)
    cap = knn.lib().tg_exact_knn_static_scratch_bytes()
    assert cap == 16 << 20
    # 8 nq k bytes beyond the scratch: refused with the sizes in the message, outputs untouched
    nq = cap // (8 * 64) + 1
    rows = torch.zeros(nq, dtype=torch.int64, device=dev)
    ids = torch.full((nq, 64), -7, dtype=torch.int32, device=dev)
    dist = torch.zeros((nq, 64), dtype=torch.float32, device=dev)
    with pytest.raises(knn.TagoreError, match="too large for the static scratch"):
        knn.exact_knn_static(X, 64, "l2", rows, out=(ids, dist))
    assert int((ids != -7).sum()) == 0
    # rows that are not a multiple of four floats would need a padded copy
    Xodd = torch.from_numpy(inputs.make("C2", n=1_000, d=30, comps=4)).to(dev)
    with pytest.raises(knn.TagoreError, match="aligned"):
        knn.exact_knn_static(Xodd, 8, "l2")
    # a row index outside the data is no query
    rows = torch.tensor([5, 4_000, -3, 17], dtype=torch.int64, device=dev)
    got = knn.exact_knn_static(X, 8, "l2", rows)
    want = knn.exact_knn(X, 8, "l2", rows[[0, 3]].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(got[0][[0, 3]], want[0]) and torch.equal(got[1][[0, 3]], want[1])
    assert int((got[0][[1, 2]] != -1).sum()) == 0 and bool(torch.isinf(got[1][[1, 2]]).all())
