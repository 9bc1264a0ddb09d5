"""Bit-reproducibility of a training step, eager and recorded into a HIP graph.

The gradient rows of a table row are summed in occurrence order (stable sort by row, fixed tree over
workgroups), so the same step gives the same bits in every run -- also from ZERO accumulators, where the
first Adagrad update is lr * sign(G) and a rounding-level difference in G would flip a whole +-lr step.
A step captured into a HIP graph (stream capture through torch) and replayed, with eager work and
synchronisations in between, must reproduce the eager step bit for bit on every replay."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar

pytestmark = pytest.mark.gpu


def _inputs(V, R, dim, B, seed):
    rng = np.random.default_rng(seed)
    ne = (rng.standard_normal((V, dim)) * 0.05).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.05).astype(np.float32)
    # half of the endpoints on five hot nodes: row segments that span many workgroups of the reduce
    hot = rng.integers(0, 5, B)
    src = np.where(rng.random(B) < 0.5, hot, rng.integers(0, V, B)).astype(np.int32)
    dst = np.where(rng.random(B) < 0.5, hot, rng.integers(0, V, B)).astype(np.int32)
    rel = rng.integers(0, R, B).astype(np.int32)
    return ne, re_, [torch.from_numpy(x).cuda() for x in (src, rel, dst)]


def _tables(tr):
    return [t.clone() for t in (tr.node_emb, tr.node_state, tr.rel_emb, tr.rel_state)]


@pytest.mark.parametrize("model,dim,B,C,N,precision", (
    (mar.MODEL_COMPLEX, 100, 2000, 4, 500, 0), (mar.MODEL_DISTMULT, 400, 3000, 3, 700, 0),
    (mar.MODEL_DISTMULT, 50, 1000, 10, 100, 0), (mar.MODEL_TRANSE, 36, 1500, 5, 300, 0),
    (mar.MODEL_COMPLEX, 100, 2000, 4, 500, 1), (mar.MODEL_DISTMULT, 400, 3000, 3, 700, 1)))
def test_same_step_twice_gives_the_same_bits(model, dim, B, C, N, precision):
    V, R = 3000, 6
    ne, re_, ids = _inputs(V, R, dim, B, seed=dim)
    results = []
    for run in range(3):
        tr = mar.Trainer(V, R, dim, model, B, C, N, N // 10, seed=5, node_emb=ne, rel_emb=re_, precision=precision)     # accumulators: zero
        for step in range(2):
            tr.sample_negatives(step, ids[0], ids[2])
            tr.train_batch(*ids)
        torch.cuda.synchronize()
        results.append((_tables(tr), tr.loss.clone()))
        tr.close()
    for tabs, loss in results[1:]:
        assert torch.equal(loss, results[0][1])
        for t, w in zip(tabs, results[0][0]):
            assert torch.equal(t, w)


@pytest.mark.parametrize("precision", (0, 1))
def test_captured_step_replays_like_the_eager_step(precision):
    V, R, dim, B, C, N = 3000, 6, 100, 2000, 4, 500
    ne, re_, ids = _inputs(V, R, dim, B, seed=0)

    def trainer():
        tr = mar.Trainer(V, R, dim, mar.MODEL_COMPLEX, B, C, N, 50, seed=5, node_emb=ne, rel_emb=re_, precision=precision)   # accumulators: zero
        tr.sample_negatives(3, ids[0], ids[2])
        return tr

    eager = trainer()
    eager.train_batch(*ids)
    torch.cuda.synchronize()
    want = _tables(eager)
    want_loss = eager.loss.clone()

    tr = trainer()
    init = _tables(tr)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            mar.mar_sample_negatives(tr.ctx, 3, ids[0], ids[2], B, tr.neg_src, tr.neg_dst)
            mar.mar_train_batch(tr.ctx, ids[0], ids[1], ids[2], B, tr.neg_src, tr.neg_dst, tr.loss, None)
    torch.cuda.synchronize()
    # capture runs nothing: the tables are still the initial ones
    assert torch.equal(tr.node_emb, init[0])
    for replay in range(3):
        for t, t0 in zip((tr.node_emb, tr.node_state, tr.rel_emb, tr.rel_state), init):
            t.copy_(t0)                                   # eager work between replays
        tr.neg_src.zero_(); tr.loss.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(tr.loss, want_loss), replay
        for t, w in zip((tr.node_emb, tr.node_state, tr.rel_emb, tr.rel_state), want):
            assert torch.equal(t, w), replay
    eager.close(); tr.close()
