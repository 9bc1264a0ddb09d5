"""GPU parity at the sizes the benchmark runs and on large id spaces (the bitmap / atomic index path,
64-bit row offsets, hot rows whose segments span many reduce tasks)."""
import numpy as np
import pytest
import torch

import synth
from oracle import sampling
from parity_util import run_step_both, run_step_device_tables, check_step

pytestmark = pytest.mark.gpu


def test_benchmark_workload_one_step_full_size():
    """kg_small exactly as bench.py runs it: first batch of the synthetic graph, sampled negatives (10% by
    degree), ComplEx d=100, 10,000 edges, 10 chunks x 1,000 negatives; every output compared."""
    w = synth.get_workload("kg_small")
    src, rel, dst = (t.numpy() for t in synth.make_graph(w.num_nodes, w.num_rels, w.num_edges, w.node_zipf, w.rel_zipf, seed=w.seed))
    ns, nd = sampling.sample_negatives(w.seed, 0, w.num_nodes, src, dst, w.num_chunks, w.negs_per_chunk, w.deg_negs_per_chunk)
    ne = sampling.init_table(w.seed, 0, w.num_nodes, w.dim, np.float32(w.init_std)).astype(np.float32)
    re_ = sampling.init_table(w.seed, 1, w.num_rels, w.dim, np.float32(w.init_std)).astype(np.float32)
    b = w.batch_size
    out = run_step_both(w.model, w.num_nodes, w.num_rels, w.dim, b, w.num_chunks, w.negs_per_chunk, b, seed=0,
                        ids=(src[:b].copy(), rel[:b].copy(), dst[:b].copy(), ns, nd), tables=(ne, re_))
    rep = check_step(out)
    print(rep, flush=True)
    # the last, short batch of the epoch (3,142 edges: 4 chunks, the last one with 142 edges)
    lo = (w.num_edges // b) * b
    out = run_step_both(w.model, w.num_nodes, w.num_rels, w.dim, b, w.num_chunks, w.negs_per_chunk, w.num_edges - lo, seed=0,
                        ids=(src[lo:].copy(), rel[lo:].copy(), dst[lo:].copy(), ns, nd), tables=(ne, re_))
    print(check_step(out), flush=True)


def _hot_ids(rng, V, R, n, C, N, hot_frac):
    """Half of the endpoints fall on a handful of hot nodes (segments of thousands of rows), the rest are
    spread over the whole id space; negatives uniform plus a share of hot ones."""
    hot = rng.integers(0, V, 5)
    def draw(m):
        ids = rng.integers(0, V, m)
        pick = rng.random(m) < hot_frac
        ids[pick] = hot[rng.integers(0, 5, pick.sum())]
        return ids.astype(np.int32)
    return (draw(n), rng.integers(0, R, n).astype(np.int32), draw(n),
            draw(C * N).reshape(C, N), draw(C * N).reshape(C, N))


def test_large_id_space_bitmap_index_and_hot_rows():
    """6 M nodes: the touched-id map is a bitmap marked with atomics; 50% of the endpoints are 5 hot nodes."""
    rng = np.random.default_rng(7)
    V, R, dim, B, C, N = 6_000_000, 3, 16, 8192, 8, 512
    ids = _hot_ids(rng, V, R, B, C, N, 0.5)
    out = run_step_device_tables(0, V, R, dim, B, C, N, ids, seed=3)
    assert out["gpu"]["untouched_ok"]
    print(check_step(out, max_flip_frac=1e-3), flush=True)


@pytest.mark.parametrize("model,precision", ((0, 0), (1, 0), (0, 1), (1, 1)))
def test_social_shape_batch_on_a_41m_row_table(model, precision):
    """Batch geometry of the social / large-KG workloads (50,000 edges, 50 chunks x 1,000 negatives, d = 100)
    on a 41.6 M-row table (16.6 GB per table, row offsets beyond 2^31 bytes); precision 1: the split-precision
    contraction in the launch configuration bench.py times (both passes split their last round)."""
    rng = np.random.default_rng(11 + model)
    V, R, dim, B, C, N = 41_600_000, (1 if model == 0 else 1000), 100, 50_000, 50, 1_000
    ids = _hot_ids(rng, V, R, B, C, N, 0.3)
    out = run_step_device_tables(model, V, R, dim, B, C, N, ids, seed=5, precision=precision)
    assert out["gpu"]["untouched_ok"]
    print(check_step(out, max_flip_frac=1e-3), flush=True)


@pytest.mark.parametrize("precision", (0, 1))
def test_large_kg_shape_with_degree_negatives_on_86m_rows(precision):
    """Geometry of the large-KG workload: 86.1 M nodes, 14,824 relations, ComplEx d = 100 (69 GB of tables and
    accumulators), 50,000 edges, 50 chunks x 1,000 negatives of which 500 are drawn by degree through the
    library's sampler from a power-law edge list (bit-exact against the oracle's sampler), then one step."""
    import paper_2101_08358_amd as mar
    w = synth.get_workload("kg_large")
    E = 4_000_000
    src, rel, dst = synth.make_graph(w.num_nodes, w.num_rels, E, w.node_zipf, w.rel_zipf, seed=1, device="cuda:0")
    es, er, ed = src.cpu().numpy(), rel.cpu().numpy(), dst.cpu().numpy()
    # negatives from the library's sampler on a small context that shares nothing but the configuration
    tr = mar.Trainer(w.num_nodes, 1, 1, 0, w.batch_size, w.num_chunks, w.negs_per_chunk, w.deg_negs_per_chunk, seed=9)
    tr.sample_negatives(123, src, dst)
    torch.cuda.synchronize()
    ns = tr.neg_src.cpu().numpy().reshape(w.num_chunks, w.negs_per_chunk)
    nd = tr.neg_dst.cpu().numpy().reshape(w.num_chunks, w.negs_per_chunk)
    tr.close()
    del tr
    torch.cuda.empty_cache()
    ons, ond = sampling.sample_negatives(9, 123, w.num_nodes, es, ed, w.num_chunks, w.negs_per_chunk, w.deg_negs_per_chunk)
    assert np.array_equal(ns, ons) and np.array_equal(nd, ond)
    b = w.batch_size
    out = run_step_device_tables(w.model, w.num_nodes, w.num_rels, w.dim, b, w.num_chunks, w.negs_per_chunk,
                                 (es[:b].copy(), er[:b].copy(), ed[:b].copy(), ons, ond), seed=2, precision=precision)
    assert out["gpu"]["untouched_ok"]
    print(check_step(out, max_flip_frac=1e-3), flush=True)


@pytest.mark.parametrize("precision", (0, 1))
def test_wide_workload_full_size_160gb(precision):
    """The wide-embedding workload at full size: 50 M nodes x 400 floats (80 GB of embeddings + 80 GB of
    accumulators), 100,000 edges, 100 chunks x 1,000 negatives; in fp32 and in split precision."""
    w = synth.get_workload("wide")
    rng = np.random.default_rng(21)
    ids = _hot_ids(rng, w.num_nodes, w.num_rels, w.batch_size, w.num_chunks, w.negs_per_chunk, 0.1)
    out = run_step_device_tables(w.model, w.num_nodes, w.num_rels, w.dim, w.batch_size, w.num_chunks, w.negs_per_chunk, ids, seed=4,
                                 precision=precision)
    assert out["gpu"]["untouched_ok"]
    print(check_step(out, max_flip_frac=1e-3), flush=True)
