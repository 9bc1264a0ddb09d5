"""GPU parity of the split-precision contraction (each fp32 operand as bf16 hi + lo, three bf16 matrix products per
product): one training step through the C ABI against the fp64 oracle, at the bars of the fp32 path."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar

from parity_util import run_step_both, check_step

pytestmark = pytest.mark.gpu

DISTMULT, COMPLEX, TRANSE, DOT = 0, 1, 2, 3
SPLIT = 1


@pytest.mark.parametrize("model", (DISTMULT, COMPLEX, DOT))
@pytest.mark.parametrize("shape", (
    # (V, R, dim, B, C, N, n_edges)
    (500, 7, 50, 1000, 10, 100, 1000),        # config-1 geometry on a small graph (heavy row reuse)
    (20000, 30, 100, 2000, 2, 1000, 2000),    # config-2/3/4 chunk geometry: several stripes, ragged tails
    (3000, 5, 100, 600, 3, 130, 470),         # ragged everything: short last chunk, N not a multiple of 16
))
def test_one_step_matches_oracle(model, shape):
    V, R, dim, B, C, N, n = shape
    print("case", model, shape, flush=True)
    out = run_step_both(model, V, R, dim, B, C, N, n, seed=100 + model, precision=SPLIT)
    print(check_step(out), flush=True)


@pytest.mark.parametrize("model,dim", ((DISTMULT, 400), (COMPLEX, 200), (DISTMULT, 36), (DISTMULT, 17), (COMPLEX, 128), (DOT, 100), (DISTMULT, 256),
                                       (DISTMULT, 144), (COMPLEX, 300), (DOT, 268)))
def test_one_step_other_widths(model, dim):
    print("case", model, dim, flush=True)
    out = run_step_both(model, 4000, 11, dim, 512, 4, 200, 512, seed=7 + dim, precision=SPLIT)
    print(check_step(out), flush=True)


@pytest.mark.parametrize("n", (1, 33))
def test_short_batches(n):
    """One edge, and one edge more than a tile of 32."""
    out = run_step_both(DISTMULT, 800, 3, 52, 256, 4, 96, n, seed=21 + n, precision=SPLIT)
    print(check_step(out), flush=True)


def test_empty_batch_is_a_no_op():
    tr = mar.Trainer(100, 2, 16, DISTMULT, 64, 2, 8, seed=3, precision=SPLIT)
    torch.cuda.synchronize()
    before = tr.node_emb.clone()
    e = torch.zeros(0, dtype=torch.int32, device=tr.device)
    tr.loss.fill_(5.0)
    tr.train_batch(e, e, e)
    torch.cuda.synchronize()
    assert tr.loss.item() == 0.0 and torch.equal(before, tr.node_emb)
    tr.close()


def test_narrowest_rows():
    out = run_step_both(DOT, 600, 1, 4, 256, 2, 64, 256, seed=2, std=0.3, precision=SPLIT)
    print(check_step(out), flush=True)


def test_ragged_chunks_at_the_widest_rows():
    """Short last chunk, chunk size and negatives not multiples of the tile, with two waves sharing each row block."""
    out = run_step_both(DISTMULT, 3000, 5, 400, 600, 3, 130, 470, seed=31, precision=SPLIT)
    print(check_step(out), flush=True)


def test_one_step_with_trained_scale_embeddings():
    """Rows of the size a trained table has (std 0.3): scores of order 10, softmax far from uniform."""
    out = run_step_both(DISTMULT, 3000, 5, 100, 1024, 4, 500, 1024, seed=3, std=0.3, precision=SPLIT)
    print(check_step(out), flush=True)


def test_one_step_when_pass_one_splits_its_last_round():
    """80 chunk-sides x 8 stripes of 128 edges = 640 units of the first pass on 512 workgroup slots: the stripes of the
    last 16 chunk-sides are split into parts over the negatives' tiles and merged afterwards."""
    out = run_step_both(DISTMULT, 50000, 3, 100, 40000, 40, 256, 40000, seed=12, precision=SPLIT)
    print(check_step(out), flush=True)


def test_one_step_when_pass_two_splits_its_last_round():
    """80 chunk-sides x 8 stripes of 128 negatives = 640 units of the second pass on 512 workgroup slots: the stripes of
    the last 16 chunk-sides are split into parts over the edges' tiles, and the parts' gradient rows added up."""
    out = run_step_both(COMPLEX, 50000, 3, 64, 40000, 40, 1024, 40000, seed=13, precision=SPLIT)
    print(check_step(out), flush=True)


def test_evaluation_in_a_split_precision_context_is_the_fp32_one():
    """Ranks are always computed in fp32: a context created for split-precision training ranks like any other."""
    rng = np.random.default_rng(9)
    V, R, dim, B, C, N = 2000, 3, 100, 512, 2, 300
    ne = (rng.standard_normal((V, dim)) * 0.3).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.3).astype(np.float32)
    ids = [torch.from_numpy(rng.integers(0, hi, B).astype(np.int32)).cuda() for hi in (V, R, V)]
    got = []
    for precision in (0, 1):
        tr = mar.Trainer(V, R, dim, mar.MODEL_COMPLEX, B, C, N, 0, node_emb=ne, rel_emb=re_, precision=precision)
        tr.sample_negatives(0)
        got.append([t.clone() for t in tr.eval_scores(*ids)])
        tr.close()
    for a, b in zip(*got):
        assert torch.equal(a, b)


def test_transe_is_refused():
    with pytest.raises(mar.MarError):
        mar.mar_workspace_bytes(mar.MarConfig(1000, 3, 50, mar.MODEL_TRANSE, 100, 10, 20, 0, 0.1, 1e-10, 0.001, 0, SPLIT, 0))


def test_single_edge_single_negative():
    check_step(run_step_both(DISTMULT, 50, 2, 50, 1, 1, 1, 1, seed=1, std=0.5, precision=SPLIT))


def test_every_edge_identical():
    """Negatives all the same node: one node row hit by everything."""
    n, C, N = 300, 3, 40
    ids = (np.full(n, 3, np.int32), np.zeros(n, np.int32), np.full(n, 4, np.int32),
           np.full((C, N), 3, np.int32), np.full((C, N), 5, np.int32))
    check_step(run_step_both(COMPLEX, 10, 1, 20, n, C, N, n, seed=2, std=0.3, ids=ids, precision=SPLIT), max_flip_frac=1.0)


def test_all_zero_tables():
    """Every score 0: loss = 2 n log N."""
    tabs = (np.zeros((60, 24), np.float32), np.zeros((3, 24), np.float32))
    out = run_step_both(DISTMULT, 60, 3, 24, 64, 2, 10, 64, seed=3, tables=tabs, precision=SPLIT)
    assert abs(out["gpu"]["loss"] - 64 * 2 * np.log(10)) < 1e-3
    check_step(out, max_flip_frac=1.0)


def test_large_scores_stay_finite_and_inside_the_products_error_bound():
    """Embeddings of size 2 (d = 50, DistMult): |q| |n| is about 400 and scores reach the hundreds.  A split-precision
    product is exact to about 2^-17 of sum_k |q_k n_k| (about 200 here), an ABSOLUTE score error of up to ~1.5e-3 that
    the exponential turns into a RELATIVE error of the softmax weights: the 1e-4 bars of the step hold while
    |q| |n| stays below about 10 (every other case here), and this case is held to 2e-3 (observed 4.5e-4)."""
    out = run_step_both(DISTMULT, 200, 3, 50, 128, 2, 50, 128, seed=4, std=2.0, precision=SPLIT)
    assert np.all(np.isfinite(out["gpu"]["node_emb"])) and np.isfinite(out["gpu"]["loss"])
    print(check_step(out, rel=2e-3, row_rel=2e-3), flush=True)


@pytest.mark.parametrize("model", (DISTMULT, COMPLEX, DOT))
def test_one_step_from_warm_state(model):
    """With accumulators of the size of G^2 the update is smooth in G: every element of the updated tables is compared."""
    from oracle import step as ostep
    from parity_util import make_tables
    rng = np.random.default_rng(5)
    V, R, dim, B, C, N = 800, 4, 100, 1000, 5, 300
    tabs = make_tables(rng, V, R, dim, 0.05)
    ns = np.full((V, dim), 0.01, np.float32); rs = np.full((R, dim), 0.01, np.float32)
    out = run_step_both(model, V, R, dim, B, C, N, B, seed=6, std=0.05, tables=tabs, node_state=ns, rel_state=rs, precision=SPLIT)
    print(check_step(out), flush=True)
    gpu, ora = out["gpu"], out["ora"]
    for k in ("node_emb", "rel_emb", "node_state", "rel_state"):
        assert np.max(np.abs(gpu[k].astype(np.float64) - ora[k])) / np.max(np.abs(ora[k])) <= 1e-4, k
