"""GPU parity: one training step through the C ABI against the oracle."""
import numpy as np
import pytest
import torch

from parity_util import run_step_both, check_step

pytestmark = pytest.mark.gpu

DISTMULT, COMPLEX, TRANSE, DOT = 0, 1, 2, 3


@pytest.mark.parametrize("model", (DISTMULT, COMPLEX, TRANSE, DOT))
@pytest.mark.parametrize("shape", (
    # (V, R, dim, B, C, N, n_edges)
    (500, 7, 50, 1000, 10, 100, 1000),        # config-1 geometry on a small graph (heavy row reuse)
    (20000, 30, 100, 2000, 2, 1000, 2000),    # config-2/3/4 chunk geometry: several 64-row stripes, ragged tails
    (3000, 5, 100, 600, 3, 130, 470),         # ragged everything: short last chunk, N not a multiple of 16
))
def test_one_step_matches_oracle(model, shape):
    V, R, dim, B, C, N, n = shape
    print("case", model, shape, flush=True)
    out = run_step_both(model, V, R, dim, B, C, N, n, seed=100 + model)
    rep = check_step(out)
    print(rep, flush=True)


@pytest.mark.parametrize("model,dim", ((DISTMULT, 400), (COMPLEX, 200), (TRANSE, 36), (DISTMULT, 17), (COMPLEX, 128), (DOT, 100)))
def test_one_step_other_widths(model, dim):
    print("case", model, dim, flush=True)
    out = run_step_both(model, 4000, 11, dim, 512, 4, 200, 512, seed=7 + dim)
    print(check_step(out), flush=True)


@pytest.mark.parametrize("model", (DISTMULT, COMPLEX, TRANSE))
def test_one_step_when_pass_one_splits_its_last_round(model):
    """96 chunk-sides x 7 stripes = 672 units of the first contraction pass on 512 workgroup slots: the stripes of
    the last 24 chunk-sides are split into two parts over the negatives' tiles and merged afterwards."""
    print("case", model, flush=True)
    out = run_step_both(model, 30000, 3, 100, 21504, 48, 128, 21504, seed=40 + model)
    print(check_step(out), flush=True)


def test_short_batch_on_a_configuration_that_splits_full_batches():
    """The same configuration with 20,000 of its 21,504 edges: short batches take no split (and leave the split's
    buffers alone)."""
    print(check_step(run_step_both(DISTMULT, 30000, 3, 100, 21504, 48, 128, 20000, seed=44)), flush=True)


@pytest.mark.parametrize("model", (DISTMULT, COMPLEX, TRANSE, DOT))
def test_one_step_from_warm_state(model):
    """With accumulators of the size of G^2 the update is smooth in G: every element is compared."""
    from oracle import step as ostep
    from parity_util import make_tables
    rng = np.random.default_rng(5)
    V, R, dim, B, C, N = 800, 4, 100, 1000, 5, 300
    tabs = make_tables(rng, V, R, dim, 0.05)
    ids = (rng.integers(0, V, B).astype(np.int32), rng.integers(0, R, B).astype(np.int32),
           rng.integers(0, V, B).astype(np.int32), rng.integers(0, V, (C, N)).astype(np.int32),
           rng.integers(0, V, (C, N)).astype(np.int32))
    dry = ostep.train_batch(model, 0.1, 1e-10, B // C, tabs[0].copy(), np.zeros_like(tabs[0]), tabs[1].copy(),
                            np.zeros_like(tabs[1]), *ids, apply_update=False)
    gn = np.max(np.abs(dry.G_nodes))
    gr = np.max(np.abs(dry.G_rels)) if dry.G_rels.size else 1.0      # Dot touches no relation row
    ns = ((rng.random((V, dim)) + 0.5) * gn * gn).astype(np.float32)
    rs = ((rng.random((R, dim)) + 0.5) * gr * gr).astype(np.float32)
    out = run_step_both(model, V, R, dim, B, C, N, B, seed=11, node_state=ns, rel_state=rs, ids=ids, tables=tabs)
    rep = check_step(out, max_flip_frac=1.0)
    gpu, ora = out["gpu"], out["ora"]
    for k in ("node_emb", "rel_emb", "node_state", "rel_state"):
        assert np.max(np.abs(gpu[k].astype(np.float64) - ora[k])) / np.max(np.abs(ora[k])) <= 1e-4, k
    if model == DOT:
        assert np.array_equal(gpu["rel_emb"], tabs[1]) and np.array_equal(gpu["rel_state"], rs)   # relations untouched
    print(rep, flush=True)


def test_degenerate_cases():
    # a single edge, a single negative, one chunk
    print("single", flush=True)
    check_step(run_step_both(DISTMULT, 50, 2, 50, 1, 1, 1, 1, seed=1, std=0.5))
    # every edge identical, negatives all the same node (one node row hit by everything)
    print("all-same", flush=True)
    n, C, N = 300, 3, 40
    ids = (np.full(n, 3, np.int32), np.zeros(n, np.int32), np.full(n, 4, np.int32),
           np.full((C, N), 3, np.int32), np.full((C, N), 5, np.int32))
    check_step(run_step_both(COMPLEX, 10, 1, 20, n, C, N, n, seed=2, std=0.3, ids=ids), max_flip_frac=1.0)
    # all-zero tables: every score 0, loss = 2 n log N, TransE distances all zero
    print("zero-tables", flush=True)
    for model in (DISTMULT, TRANSE):
        tabs = (np.zeros((60, 24), np.float32), np.zeros((3, 24), np.float32))
        out = run_step_both(model, 60, 3, 24, 64, 2, 10, 64, seed=3, tables=tabs)
        assert abs(out["gpu"]["loss"] - 64 * 2 * np.log(10)) < 1e-3
        check_step(out, max_flip_frac=1.0)
    # large scores: the softmax must not overflow
    print("large-scores", flush=True)
    out = run_step_both(DISTMULT, 200, 3, 50, 128, 2, 50, 128, seed=4, std=2.0)
    assert np.all(np.isfinite(out["gpu"]["node_emb"])) and np.isfinite(out["gpu"]["loss"])
    check_step(out)


def test_many_contexts_created_and_destroyed():
    """Every context owns a stream and a few events: creating and destroying many in a row, in both precisions and with
    a step in between, must leave nothing behind and keep giving the same step."""
    import paper_2101_08358_amd as mar
    rng = np.random.default_rng(0)
    ne = (rng.standard_normal((300, 32)) * 0.1).astype(np.float32)
    re_ = (rng.standard_normal((2, 32)) * 0.1).astype(np.float32)
    ids = [torch.from_numpy(rng.integers(0, hi, 64).astype(np.int32)).cuda() for hi in (300, 2, 300)]
    want = {}
    for i in range(120):
        precision = i % 2
        tr = mar.Trainer(300, 2, 32, DISTMULT, 64, 2, 16, seed=1, node_emb=ne, rel_emb=re_, precision=precision)
        tr.sample_negatives(0)
        tr.train_batch(*ids)
        torch.cuda.synchronize()
        got = (tr.node_emb.clone(), float(tr.loss.item()))
        tr.close()
        if precision not in want:
            want[precision] = got
        assert got[1] == want[precision][1] and torch.equal(got[0], want[precision][0])


def test_empty_batch_is_a_no_op():
    import paper_2101_08358_amd as mar
    tr = mar.Trainer(100, 2, 16, DISTMULT, 64, 2, 8, seed=3)
    torch.cuda.synchronize()
    before = tr.node_emb.clone()
    e = torch.zeros(0, dtype=torch.int32, device=tr.device)
    tr.loss.fill_(5.0)
    tr.train_batch(e, e, e)
    torch.cuda.synchronize()
    assert tr.loss.item() == 0.0 and torch.equal(before, tr.node_emb)
    tr.close()


@pytest.mark.parametrize("level", (1e-2, 1e-3, 1e-4))
def test_transe_negatives_that_nearly_coincide_with_the_target(level):
    """TransE: negatives placed at s + r + delta (destination side) and d - r + delta (source side) with
    |delta| / |s + r| = level, where the expansion |q|^2 + |n|^2 - 2 q.n of the squared distance cancels to its
    last bits.  Scores, log-sum-exp, loss and the gradient tensors must still meet the 1e-4 bars, and so must
    every single gradient row down to level 1e-3.  At 1e-4 the row bar is what fp32 operands allow: the kernel
    forms q = s + r in fp32 (rounding 2^-24 |q_k| per component) while delta's components are level * |q_k|, so
    the direction (q - n) / |q - n| of the near pair's gradient term is only known to about 2^-23 / level (measured
    on the host: 4e-4 median, 9e-4 worst at this level); the oracle takes the same fp32 inputs to fp64 first."""
    rng = np.random.default_rng(int(-np.log10(level)))
    V, R, dim, B, C, N = 2000, 5, 100, 512, 4, 200
    S = B // C
    ne = (rng.standard_normal((V, dim)) * 0.05).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.05).astype(np.float32)
    src = rng.integers(0, V - 200, B).astype(np.int32)
    rel = rng.integers(0, R, B).astype(np.int32)
    dst = rng.integers(0, V - 200, B).astype(np.int32)
    neg_src = rng.integers(0, V - 200, (C, N)).astype(np.int32)
    neg_dst = rng.integers(0, V - 200, (C, N)).astype(np.int32)
    spare = V - 200                                               # rows V-200.. are rewritten as near-coincident negatives
    for c in range(C):
        for k in range(12):                                       # 12 edges per chunk and side get such a negative
            e = c * S + 7 * k
            delta = rng.standard_normal(dim)
            q = ne[src[e]].astype(np.float64) + re_[rel[e]]
            ne[spare] = (q + delta / np.linalg.norm(delta) * level * np.linalg.norm(q)).astype(np.float32)
            neg_dst[c, 3 * k] = spare; spare += 1
            delta = rng.standard_normal(dim)
            q = ne[dst[e]].astype(np.float64) - re_[rel[e]]
            ne[spare] = (q + delta / np.linalg.norm(delta) * level * np.linalg.norm(q)).astype(np.float32)
            neg_src[c, 3 * k + 1] = spare; spare += 1
    out = run_step_both(TRANSE, V, R, dim, B, C, N, B, seed=0, tables=(ne, re_), ids=(src, rel, dst, neg_src, neg_dst))
    # the near-coincident negatives are the best-scoring ones of their edges
    res = out["ora"]["res"]
    assert np.all(res.lse_dst[::7][:12] > -10 * level * 1.0)
    print(check_step(out, row_rel=max(1e-4, 2.0 ** -23 / level)), flush=True)
