"""A training step recorded into a HIP graph (stream capture through torch) and replayed: every replay,
with eager work and synchronisations in between, must reproduce the eager step."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_the_eager_step():
    rng = np.random.default_rng(0)
    V, R, dim, B, C, N = 3000, 6, 100, 2000, 4, 500
    ne = (rng.standard_normal((V, dim)) * 0.05).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.05).astype(np.float32)
    ids = [torch.from_numpy(rng.integers(0, hi, B).astype(np.int32)).cuda() for hi in (V, R, V)]

    def trainer():
        # non-zero accumulators: the update is then smooth in the gradient, so two runs that sum a row's
        # gradient in different orders agree to rounding (from zero it would be lr * sign(G))
        tr = mar.Trainer(V, R, dim, mar.MODEL_COMPLEX, B, C, N, 50, seed=5, node_emb=ne, rel_emb=re_,
                         node_state=np.full((V, dim), 1e-2, np.float32), rel_state=np.full((R, dim), 1e-2, np.float32))
        tr.sample_negatives(3, ids[0], ids[2])
        return tr

    eager = trainer()
    eager.train_batch(*ids)
    torch.cuda.synchronize()
    want = [t.clone() for t in (eager.node_emb, eager.node_state, eager.rel_emb, eager.rel_state)]
    want_loss = eager.loss.item()

    tr = trainer()
    init = [t.clone() for t in (tr.node_emb, tr.node_state, tr.rel_emb, tr.rel_state)]
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
        assert abs(tr.loss.item() - want_loss) <= 1e-5 * abs(want_loss), replay
        for t, w in zip((tr.node_emb, tr.node_state, tr.rel_emb, tr.rel_state), want):
            err = (t.double() - w.double()).abs().max().item()
            # summation order inside a row's segment may differ between runs: equal up to rounding
            assert err <= 1e-5 * w.abs().max().item(), (replay, err)
    eager.close(); tr.close()
