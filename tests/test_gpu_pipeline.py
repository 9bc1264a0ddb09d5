"""Out-of-memory pipelined training (Sec. 3) through the C ABI: node table and accumulators in pinned host memory.
depth 1 must reproduce the resident step bit for bit; depth k must follow the oracle's bounded-staleness loop with
staleness k - 1 (and give the same bits in every run: the stage order is fixed by events, not by timing)."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar
from oracle import pipeline as opipe

pytestmark = pytest.mark.gpu


def _setup(model, V, R, dim, B, C, N, nb, seed, hot=0.3, state0=0.0):
    rng = np.random.default_rng(seed)
    ne = (rng.standard_normal((V, dim)) * 0.05).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.05).astype(np.float32)
    ns = np.full((V, dim), state0, np.float32)
    rs = np.full((R, dim), state0, np.float32)
    batches = []
    for _ in range(nb):
        n = B if len(batches) % 3 else B - 37                      # a short batch now and then
        pick = lambda m: np.where(rng.random(m) < hot, rng.integers(0, 8, m), rng.integers(0, V, m)).astype(np.int32)
        batches.append((pick(n), rng.integers(0, R, n).astype(np.int32), pick(n),
                        rng.integers(0, V, (C, N)).astype(np.int32), rng.integers(0, V, (C, N)).astype(np.int32)))
    return ne, ns, re_, rs, batches


def _run_pipe(model, V, R, dim, B, C, N, depth, tables, batches, side_stream=True, precision=0):
    ne, ns, re_, rs = tables
    dev = torch.device("cuda:0")
    h_ne = torch.from_numpy(ne.copy()).pin_memory()
    h_ns = torch.from_numpy(ns.copy()).pin_memory()
    d_re = torch.from_numpy(re_.copy()).to(dev)
    d_rs = torch.from_numpy(rs.copy()).to(dev)
    cfg = mar.MarConfig(V, R, dim, model, B, C, N, 0, 0.1, 1e-10, 0.001, 0, precision, 0)
    nbytes = mar.mar_pipe_workspace_bytes(cfg, depth)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    pipe = mar.mar_pipe_create(cfg, h_ne, h_ns, d_re, d_rs, ws, nbytes, depth)
    # ids of all batches go to the device up front, on a side stream: the staging stage waits for that stream only
    ids_stream = torch.cuda.Stream() if side_stream else torch.cuda.current_stream()
    with torch.cuda.stream(ids_stream):
        dbs = [[torch.from_numpy(x.reshape(-1)).to(dev) for x in bt] for bt in batches]
    losses = torch.zeros(len(batches), dtype=torch.float32, device=dev)
    for j, (bt, db) in enumerate(zip(batches, dbs)):
        mar.mar_pipe_submit(pipe, db[0], db[1], db[2], bt[0].shape[0], db[3], db[4], losses[j:j + 1], ids_stream=ids_stream)
    mar.mar_pipe_drain(pipe)
    torch.cuda.synchronize()
    out = (h_ne.numpy().copy(), h_ns.numpy().copy(), d_re.cpu().numpy(), d_rs.cpu().numpy(), losses.cpu().numpy())
    mar.mar_pipe_destroy(pipe)
    return out


def _run_resident(model, V, R, dim, B, C, N, tables, batches, precision=0):
    ne, ns, re_, rs = tables
    tr = mar.Trainer(V, R, dim, model, B, C, N, 0, 0.1, 1e-10, 0.001, 0, node_emb=ne, rel_emb=re_, node_state=ns, rel_state=rs,
                     precision=precision)
    losses = []
    for bt in batches:
        tr.neg_src.copy_(torch.from_numpy(bt[3].reshape(-1))); tr.neg_dst.copy_(torch.from_numpy(bt[4].reshape(-1)))
        tr.train_batch(*(torch.from_numpy(x).to(tr.device) for x in bt[:3]))
        losses.append(tr.loss.clone())
    torch.cuda.synchronize()
    out = (tr.node_emb.cpu().numpy(), tr.node_state.cpu().numpy(), tr.rel_emb.cpu().numpy(), tr.rel_state.cpu().numpy(),
           torch.cat(losses).cpu().numpy())
    tr.close()
    return out


@pytest.mark.parametrize("model,dim", ((mar.MODEL_COMPLEX, 100), (mar.MODEL_DISTMULT, 50), (mar.MODEL_DOT, 36), (mar.MODEL_TRANSE, 17)))
def test_depth_one_is_the_resident_step_bit_for_bit(model, dim):
    V, R, B, C, N = 5000, 6, 600, 3, 200
    ne, ns, re_, rs, batches = _setup(model, V, R, dim, B, C, N, nb=5, seed=dim)
    got = _run_pipe(model, V, R, dim, B, C, N, 1, (ne, ns, re_, rs), batches)
    want = _run_resident(model, V, R, dim, B, C, N, (ne, ns, re_, rs), batches)
    for g, w, name in zip(got, want, ("node_emb", "node_state", "rel_emb", "rel_state", "loss")):
        assert np.array_equal(g, w), name


def test_depth_one_is_the_resident_step_in_split_precision():
    model, dim, V, R, B, C, N = mar.MODEL_COMPLEX, 100, 5000, 6, 600, 3, 200
    ne, ns, re_, rs, batches = _setup(model, V, R, dim, B, C, N, nb=4, seed=11)
    got = _run_pipe(model, V, R, dim, B, C, N, 1, (ne, ns, re_, rs), batches, precision=1)
    want = _run_resident(model, V, R, dim, B, C, N, (ne, ns, re_, rs), batches, precision=1)
    for g, w, name in zip(got, want, ("node_emb", "node_state", "rel_emb", "rel_state", "loss")):
        assert np.array_equal(g, w), name


def test_depth_one_is_the_resident_step_when_pass_one_splits_its_last_round():
    """A batch large enough for the first contraction pass to split the stripes beyond its last whole round of
    workgroups (96 chunk-sides x 7 stripes = 672 units on 512 slots): the merge of the parts belongs to the step
    wherever the step is launched from."""
    model, V, R, dim, B, C, N = mar.MODEL_DISTMULT, 30000, 3, 100, 21504, 48, 128
    ne, ns, re_, rs, batches = _setup(model, V, R, dim, B, C, N, nb=3, seed=7, hot=0.05)
    batches = [bt if bt[0].shape[0] == B else tuple(np.resize(x, B) if i < 3 else x for i, x in enumerate(bt)) for bt in batches]
    got = _run_pipe(model, V, R, dim, B, C, N, 1, (ne, ns, re_, rs), batches)
    want = _run_resident(model, V, R, dim, B, C, N, (ne, ns, re_, rs), batches)
    for g, w, name in zip(got, want, ("node_emb", "node_state", "rel_emb", "rel_state", "loss")):
        assert np.array_equal(g, w), name
    # the first step's loss from tables of size 0.05: near 2 log N per edge, and the same number both ways
    assert abs(want[4][0] / B - 2 * np.log(N)) < 0.5


@pytest.mark.parametrize("depth", (2, 4))
def test_depth_k_follows_the_oracle_with_staleness_k_minus_one(depth):
    """Warm accumulators (of the size of the squared gradients) make the update smooth in the gradient, so tables can
    be compared directly; hot nodes shared by consecutive batches make stale reads matter."""
    model, V, R, dim, B, C, N = mar.MODEL_COMPLEX, 3000, 5, 100, 500, 5, 100
    ne, ns, re_, rs, batches = _setup(model, V, R, dim, B, C, N, nb=7, seed=depth, state0=0.05)
    got = _run_pipe(model, V, R, dim, B, C, N, depth, (ne, ns, re_, rs), batches)
    again = _run_pipe(model, V, R, dim, B, C, N, depth, (ne, ns, re_, rs), batches)
    for g, a in zip(got, again):
        assert np.array_equal(g, a)                                 # same bits in every run
    one, ons, ore, ors = ne.copy(), ns.copy(), re_.copy(), rs.copy()
    ol = opipe.train_pipelined(model, np.float32(0.1), np.float32(1e-10), B // C, one, ons, ore, ors, batches, staleness=depth - 1)
    for g, w, name in zip(got[:4], (one, ons, ore, ors), ("node_emb", "node_state", "rel_emb", "rel_state")):
        err = np.max(np.abs(g.astype(np.float64) - w)) / np.max(np.abs(w))
        assert err <= 1e-4, (name, err)
    assert np.max(np.abs(got[4] - np.array(ol)) / np.abs(np.array(ol))) <= 1e-4
    # and staleness matters here: the synchronous loop ends somewhere else
    sne, sns, sre, srs = ne.copy(), ns.copy(), re_.copy(), rs.copy()
    opipe.train_pipelined(model, np.float32(0.1), np.float32(1e-10), B // C, sne, sns, sre, srs, batches, staleness=0)
    assert np.max(np.abs(sne - one)) / np.max(np.abs(one)) > 1e-3
