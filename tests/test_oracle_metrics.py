"""Pins for the oracle's MRR / Hits@k: closed forms and a plain loop."""
import math

import numpy as np

from oracle import metrics


def test_closed_forms():
    n = 50
    assert metrics.mrr(np.ones(n, int)) == 1.0 and metrics.hits_at(np.ones(n, int), 1) == 1.0
    r = np.arange(1, n + 1)
    harmonic = sum(1.0 / k for k in range(1, n + 1))
    assert math.isclose(metrics.mrr(r), harmonic / n, rel_tol=1e-15)
    for k in (1, 3, 10, 50, 80):
        assert math.isclose(metrics.hits_at(r, k), min(k, n) / n)
    assert metrics.mrr(np.full(7, 4)) == 0.25 and metrics.hits_at(np.full(7, 4), 3) == 0.0
    assert metrics.hits_at(np.full(7, 4), 4) == 1.0          # the threshold is inclusive
    assert metrics.mrr([]) == 0.0 and metrics.hits_at([], 10) == 0.0


def test_against_plain_loop():
    rng = np.random.default_rng(0)
    r = rng.integers(1, 1002, 5000)
    s = 0.0
    h = {1: 0, 10: 0, 100: 0}
    for x in r.tolist():
        s += 1.0 / x
        for k in h:
            h[k] += x <= k
    assert math.isclose(metrics.mrr(r), s / r.size, rel_tol=1e-13)
    for k, c in h.items():
        assert metrics.hits_at(r, k) == c / r.size
    # permutation invariance and monotonicity in k
    assert math.isclose(metrics.mrr(rng.permutation(r)), metrics.mrr(r), rel_tol=1e-13)
    assert metrics.hits_at(r, 1) <= metrics.hits_at(r, 10) <= metrics.hits_at(r, 100) <= 1.0
