"""The bounded hand-over of candidates that the device build uses, against the plain method, on the CPU.

The plain method is O-NND's reference mode (section 3.1.1 steps 1-3, Algorithm 1: every evaluated pair is offered to
both nodes, unbounded candidate lists, one update per round).  The model of the device build keeps, per member and
group of eight block positions, the closest candidate the member does not list yet, hands it over through C hashed
slots and updates the lists after every part of a round.  Both run the same number of rounds from the same random
lists; the recall of the model must stay within 0.005 of the plain method's.
"""
import numpy as np
import pytest

import oracle
from paper_2508_08744_amd import inputs, knn


def _recalls(X, k, metric, seed, iters, rows, truth):
    prm = knn.default_params(k, iters, metric=metric, seed=seed)
    out = []
    for kw in (dict(S=prm.S, R=prm.R, m=prm.m, seed=seed), oracle.device_model(prm)):
        o = oracle.NNDescent(X, k, metric, **kw)
        o.run(prm.it1, prm.it2)
        out.append(oracle.recall(o.graph()[0][rows], truth))
    return out


@pytest.mark.parametrize("cfg,n", [("C1", 6000), ("C2", 20000)])
def test_default_hand_over_is_within_0_005_of_the_plain_method(cfg, n):
    c = inputs.CONFIGS[cfg]
    k, metric = c["k"], oracle.METRIC_L2
    X = inputs.make(cfg, n=n)
    rows = inputs.sample_rows(n, 1000, seed=4)
    truth, _ = oracle.brute_force_knn(X, k, metric, rows)
    gaps = []
    for seed in (1, 2, 3):
        plain, model = _recalls(X, k, metric, seed, 4, rows, truth)
        assert plain > 0.99                      # (four rounds converge at these sizes)
        gaps.append(model - plain)
    print("%s n=%d: recall(model) - recall(plain) after 4 rounds, seeds 1-3: %s" % (cfg, n, " ".join("%+.4f" % g for g in gaps)))
    assert min(gaps) >= -0.005, gaps
