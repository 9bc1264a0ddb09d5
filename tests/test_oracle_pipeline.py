"""Pins of the oracle's bounded-staleness training loop (Sec. 3: pipeline stages, "Bounded Staleness")."""
import numpy as np
import pytest

from oracle import pipeline, step as ostep

LR, EPS = np.float32(0.1), np.float32(1e-10)


def _tables(rng, V, R, dim, std=0.05):
    return ((rng.standard_normal((V, dim)) * std).astype(np.float32), np.zeros((V, dim), np.float32),
            (rng.standard_normal((R, dim)) * std).astype(np.float32), np.zeros((R, dim), np.float32))


def _batches(rng, V, R, nb, B, C, N, lo=0, hi=None):
    hi = V if hi is None else hi
    out = []
    for _ in range(nb):
        out.append((rng.integers(lo, hi, B).astype(np.int32), rng.integers(0, R, B).astype(np.int32),
                    rng.integers(lo, hi, B).astype(np.int32), rng.integers(lo, hi, (C, N)).astype(np.int32),
                    rng.integers(lo, hi, (C, N)).astype(np.int32)))
    return out


@pytest.mark.parametrize("model", (0, 1, 2, 3))
def test_staleness_zero_is_the_synchronous_loop(model):
    """s = 0: every batch sees all earlier updates: bit-identical to calling the synchronous step in a loop (Alg. 1)."""
    rng = np.random.default_rng(model)
    V, R, dim, B, C, N = 60, 3, 8, 12, 3, 5
    t0 = _tables(rng, V, R, dim)
    batches = _batches(rng, V, R, 5, B, C, N)
    a = [x.copy() for x in t0]
    la = pipeline.train_pipelined(model, LR, EPS, B // C, *a, batches, staleness=0)
    b = [x.copy() for x in t0]
    lb = [ostep.train_batch(model, LR, EPS, B // C, *b, *bt).loss_sum for bt in batches]
    assert la == lb
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_stale_reads_do_not_matter_when_batches_in_flight_share_no_node():
    """Batches j and j+1 touch disjoint node ranges: a node row read by batch j+1 cannot have been changed by batch j,
    so staleness 1 gives exactly the tables of the synchronous loop (relations, shared by all, are never stale)."""
    rng = np.random.default_rng(7)
    V, R, dim, B, C, N = 90, 2, 6, 10, 2, 4
    t0 = _tables(rng, V, R, dim)
    batches = []
    for j in range(6):
        lo = 30 * (j % 3)
        batches += _batches(rng, V, R, 1, B, C, N, lo, lo + 30)
    a = [x.copy() for x in t0]
    la = pipeline.train_pipelined(0, LR, EPS, B // C, *a, batches, staleness=1)
    b = [x.copy() for x in t0]
    lb = pipeline.train_pipelined(0, LR, EPS, B // C, *b, batches, staleness=0)
    assert la == lb
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # with staleness 2 batch j+2 (same node range as j... no: j+3 shares j's range) still agrees; staleness 3 does not
    c = [x.copy() for x in t0]
    pipeline.train_pipelined(0, LR, EPS, B // C, *c, batches, staleness=2)
    assert all(np.array_equal(x, y) for x, y in zip(c, b))
    d = [x.copy() for x in t0]
    pipeline.train_pipelined(0, LR, EPS, B // C, *d, batches, staleness=3)
    assert not np.array_equal(d[0], b[0])


def test_two_batches_by_hand():
    """Two single-edge batches that share their source node, staleness 1.  Batch 1 must differentiate at the INITIAL
    node rows (batch 0's node update is still in flight) but at the UPDATED relation row, and its node gradient is then
    applied with Adagrad to the rows batch 0 has already changed: accumulator = G0^2 + G1^2 on the shared node."""
    rng = np.random.default_rng(3)
    V, R, dim = 6, 1, 4
    ne, ns, re_, rs = _tables(rng, V, R, dim, std=0.5)
    b0 = (np.array([0], np.int32), np.array([0], np.int32), np.array([1], np.int32), np.array([[4]], np.int32), np.array([[5]], np.int32))
    b1 = (np.array([0], np.int32), np.array([0], np.int32), np.array([2], np.int32), np.array([[3]], np.int32), np.array([[5]], np.int32))
    # by hand, from the pinned synchronous step's gradients
    g0 = ostep.train_batch(0, LR, EPS, 1, ne, ns, re_, rs, *b0, apply_update=False)
    re1, rs1 = re_.copy(), rs.copy()
    ostep.adagrad_rows(re1, rs1, g0.uniq_rels.astype(np.int64), g0.G_rels, LR, EPS)
    g1 = ostep.train_batch(0, LR, EPS, 1, ne, ns, re1, rs1, *b1, apply_update=False)        # initial nodes, updated relation
    ne_x, ns_x = ne.copy(), ns.copy()
    ostep.adagrad_rows(ne_x, ns_x, g0.uniq_nodes.astype(np.int64), g0.G_nodes, LR, EPS)
    ostep.adagrad_rows(ne_x, ns_x, g1.uniq_nodes.astype(np.int64), g1.G_nodes, LR, EPS)
    i0 = list(g0.uniq_nodes).index(0); i1 = list(g1.uniq_nodes).index(0)
    assert np.allclose(ns_x[0], g0.G_nodes[i0] ** 2 + g1.G_nodes[i1] ** 2, rtol=1e-6)
    a = [ne.copy(), ns.copy(), re_.copy(), rs.copy()]
    losses = pipeline.train_pipelined(0, LR, EPS, 1, *a, [b0, b1], staleness=1)
    assert losses == [g0.loss_sum, g1.loss_sum]
    assert np.array_equal(a[0], ne_x) and np.array_equal(a[1], ns_x)
    # and it differs from the synchronous result, where batch 1 sees node 0 after batch 0's update
    s = [ne.copy(), ns.copy(), re_.copy(), rs.copy()]
    pipeline.train_pipelined(0, LR, EPS, 1, *s, [b0, b1], staleness=0)
    assert not np.array_equal(s[0][0], a[0][0])
