"""GPU parity: link-prediction scores and ranks against the oracle."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar
from oracle import step as ostep

pytestmark = pytest.mark.gpu


def _run(model, V, R, dim, B, C, N, n, seed, std=0.3, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        ne = rng.integers(-2, 3, (V, dim)).astype(np.float32)
        re_ = rng.integers(-2, 3, (R, dim)).astype(np.float32)
    else:
        ne = (rng.standard_normal((V, dim)) * std).astype(np.float32)
        re_ = (rng.standard_normal((R, dim)) * std).astype(np.float32)
    src, rel, dst = (rng.integers(0, V, n).astype(np.int32), rng.integers(0, R, n).astype(np.int32),
                     rng.integers(0, V, n).astype(np.int32))
    neg_src, neg_dst = rng.integers(0, V, (C, N)).astype(np.int32), rng.integers(0, V, (C, N)).astype(np.int32)
    tr = mar.Trainer(V, R, dim, model, B, C, N, node_emb=ne, rel_emb=re_)
    tr.neg_src.copy_(torch.from_numpy(neg_src.reshape(-1))); tr.neg_dst.copy_(torch.from_numpy(neg_dst.reshape(-1)))
    pos, rd, rs = tr.eval_scores(*(torch.from_numpy(x).to(tr.device) for x in (src, rel, dst)))
    torch.cuda.synchronize()
    got = pos.cpu().numpy(), rd.cpu().numpy(), rs.cpu().numpy()
    assert torch.equal(tr.node_emb.cpu(), torch.from_numpy(ne))      # tables untouched
    tr.close()
    exp = ostep.eval_scores(model, B // C, ne, re_, src, rel, dst, neg_src, neg_dst, return_blocks=True)
    return got, exp


@pytest.mark.parametrize("model", (0, 1, 2, 3))
def test_ranks_exact_on_integer_embeddings(model):
    """Small-integer embeddings make every score's decisive quantity exact in fp32 and fp64 (the sum for
    DistMult / ComplEx, the squared distance for TransE, whose square root is monotone), ties included (a
    negative equal to the edge's own endpoint); ranks must then agree exactly."""
    got, exp = _run(model, 60, 3, 24, 300, 3, 70, 260, seed=model, integer=True)
    if model != 2:
        assert np.array_equal(got[0], exp[0].astype(np.float32))
    else:
        assert np.allclose(got[0], exp[0], rtol=1e-6)
    assert np.array_equal(got[1], exp[1]) and np.array_equal(got[2], exp[2])


def _tolerant(got, exp, S):
    """A rank is an integer decided by float comparisons: where a negative's score is within rounding of
    the positive's, either outcome is valid.  The rank must lie between the counts with the margin
    subtracted and added."""
    pos, rd, rs, blocks = exp
    assert np.max(np.abs(got[0] - pos)) <= 1e-4 * max(np.max(np.abs(pos)), 1e-30)
    n = pos.shape[0]
    decided = 0
    for side, ranks, oranks in ((0, got[1], rd), (1, got[2], rs)):
        for c, blk in enumerate(blocks):
            A = blk[side]
            lo, hi = c * S, c * S + A.shape[0]
            tol = 2e-6 * max(np.max(np.abs(A)), np.max(np.abs(pos)))
            rmin = 1 + np.sum(A > pos[lo:hi, None] + tol, axis=1)
            rmax = 1 + np.sum(A > pos[lo:hi, None] - tol, axis=1)
            assert np.all(ranks[lo:hi] >= rmin) and np.all(ranks[lo:hi] <= rmax)
            # where no negative is within the margin (no collision with the edge's own endpoint, no
            # near tie) the rank is unique and must equal the oracle's
            sure = rmin == rmax
            assert np.array_equal(ranks[lo:hi][sure], oranks[lo:hi][sure])
            decided += int(sure.sum())
    assert decided >= 0.5 * 2 * n


@pytest.mark.parametrize("model", (0, 1, 2, 3))
@pytest.mark.parametrize("shape", ((5000, 9, 100, 2000, 2, 1000, 1700), (300, 2, 50, 100, 10, 100, 100),
                                   (2000, 3, 400, 512, 2, 300, 500), (2000, 3, 128, 512, 2, 300, 500)))
def test_ranks_within_rounding_of_oracle(model, shape):
    V, R, dim, B, C, N, n = shape
    got, exp = _run(model, V, R, dim, B, C, N, n, seed=10 + model)
    _tolerant(got, exp, B // C)
    assert got[1].min() >= 1 and got[1].max() <= N + 1


def test_mrr_and_hits_from_gpu_ranks():
    """Ranks -> MRR / Hits@k on the device against the oracle's reduction of the same ranks: hit counts are
    integers (exact), the reciprocal sum is fp64 on both sides."""
    from oracle import metrics
    rng = np.random.default_rng(3)
    V, R, dim, B, C, N, n = 4000, 5, 50, 1000, 10, 100, 940
    ne = (rng.standard_normal((V, dim)) * 0.3).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.3).astype(np.float32)
    tr = mar.Trainer(V, R, dim, 0, B, C, N, node_emb=ne, rel_emb=re_)
    tr.sample_negatives(5)
    ids = [torch.from_numpy(rng.integers(0, hi, n).astype(np.int32)).to(tr.device) for hi in (V, R, V)]
    pos, rd, rs = tr.eval_scores(*ids)
    both = torch.cat([rd, rs]).contiguous()
    ks = [1, 3, 10, 50]
    out = torch.zeros(1 + len(ks), dtype=torch.float64, device=tr.device)
    mar.mar_rank_metrics(tr.ctx, both, both.numel(), ks, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ranks = both.cpu().numpy()
    assert abs(got[0] - metrics.mrr(ranks)) <= 1e-12
    for j, k in enumerate(ks):
        assert got[1 + j] == metrics.hits_at(ranks, k)
    # degenerate sizes
    mar.mar_rank_metrics(tr.ctx, both, 0, ks, out)
    torch.cuda.synchronize()
    assert torch.count_nonzero(out).item() == 0
    one = torch.tensor([7], dtype=torch.int32, device=tr.device)
    mar.mar_rank_metrics(tr.ctx, one, 1, [7], out)
    torch.cuda.synchronize()
    assert out[0].item() == 1.0 / 7 and out[1].item() == 1.0
    tr.close()


@pytest.mark.parametrize("model", (0, 1, 2, 3))
def test_filtered_ranks_against_oracle(model):
    """All nodes as negatives, then the other true edges filtered out; small-integer embeddings make every
    comparison exact, so the ranks must equal the oracle's."""
    rng = np.random.default_rng(40 + model)
    V, R, dim, n = 120, 3, 24, 90
    ne = rng.integers(-2, 3, (V, dim)).astype(np.float32)
    re_ = rng.integers(-2, 3, (R, dim)).astype(np.float32)
    true_edges = [(int(rng.integers(V)), int(rng.integers(R)), int(rng.integers(V))) for _ in range(1500)]
    true_edges = sorted(set(true_edges))
    src, rel, dst = (np.array(x, dtype=np.int32) for x in zip(*true_edges[:n]))
    # per eval edge: the other true destinations of (s, r, .) and the other true sources of (., r, d)
    by_sr, by_rd = {}, {}
    for s_, r_, d_ in true_edges:
        by_sr.setdefault((s_, r_), []).append(d_)
        by_rd.setdefault((r_, d_), []).append(s_)
    dlist = [[c for c in by_sr[(s_, r_)] if c != d_] for s_, r_, d_ in zip(src, rel, dst)]
    slist = [[c for c in by_rd[(r_, d_)] if c != s_] for s_, r_, d_ in zip(src, rel, dst)]
    csr = lambda ls: (np.concatenate([[0], np.cumsum([len(x) for x in ls])]).astype(np.int64),
                      np.array([c for x in ls for c in x] or [0], dtype=np.int32))
    (doff, dids), (soff, sids) = csr(dlist), csr(slist)
    assert doff[-1] > 0 and soff[-1] > 0
    # one chunk whose negatives are all nodes
    tr = mar.Trainer(V, R, dim, model, n, 1, V, node_emb=ne, rel_emb=re_)
    allnodes = torch.arange(V, dtype=torch.int32, device=tr.device)
    tr.neg_src.copy_(allnodes); tr.neg_dst.copy_(allnodes)
    d_ids = [torch.from_numpy(x).to(tr.device) for x in (src, rel, dst)]
    pos, rd, rs = tr.eval_scores(*d_ids)
    dev = lambda x: torch.from_numpy(x).to(tr.device)
    mar.mar_eval_filter(tr.ctx, d_ids[0], d_ids[1], d_ids[2], n, dev(doff), dev(dids), dev(soff), dev(sids), pos, rd, rs)
    torch.cuda.synchronize()
    ed, es = ostep.filtered_ranks(model, ne, re_, src, rel, dst, true_edges)
    assert np.array_equal(rd.cpu().numpy(), ed) and np.array_equal(rs.cpu().numpy(), es)
    tr.close()


@pytest.mark.parametrize("model", (0, 1, 2, 3))
def test_filtered_ranks_on_real_valued_embeddings(model):
    """The same filtered evaluation on N(0, 0.3^2) embeddings.  A rank is an integer decided by float
    comparisons: where a candidate's score is within rounding of the edge's, either outcome is valid, so the
    GPU rank must lie between the fp64 counts taken with the margin subtracted and added (and is never below
    1); where no candidate is within the margin the rank is unique and must equal the oracle's."""
    from oracle import models
    rng = np.random.default_rng(140 + model)
    V, R, dim, n = 300, 3, 100, 120
    ne = (rng.standard_normal((V, dim)) * 0.3).astype(np.float32)
    re_ = (rng.standard_normal((R, dim)) * 0.3).astype(np.float32)
    # a few nodes are near copies of others (relative distance 1e-6): candidates within rounding of the edge
    ne[V - 10:] = ne[:10] * np.float32(1 + 1e-6)
    true_edges = sorted(set((int(rng.integers(V)), int(rng.integers(R)), int(rng.integers(V))) for _ in range(6000)))
    src, rel, dst = (np.array(x, dtype=np.int32) for x in zip(*true_edges[:n]))
    by_sr, by_rd = {}, {}
    for s_, r_, d_ in true_edges:
        by_sr.setdefault((s_, r_), []).append(d_)
        by_rd.setdefault((r_, d_), []).append(s_)
    dlist = [[c for c in by_sr[(s_, r_)] if c != d_] for s_, r_, d_ in zip(src, rel, dst)]
    slist = [[c for c in by_rd[(r_, d_)] if c != s_] for s_, r_, d_ in zip(src, rel, dst)]
    csr = lambda ls: (np.concatenate([[0], np.cumsum([len(x) for x in ls])]).astype(np.int64),
                      np.array([c for x in ls for c in x] or [0], dtype=np.int32))
    (doff, dids), (soff, sids) = csr(dlist), csr(slist)
    assert doff[-1] > 0 and soff[-1] > 0
    tr = mar.Trainer(V, R, dim, model, n, 1, V, node_emb=ne, rel_emb=re_)
    allnodes = torch.arange(V, dtype=torch.int32, device=tr.device)
    tr.neg_src.copy_(allnodes); tr.neg_dst.copy_(allnodes)
    d_ids = [torch.from_numpy(x).to(tr.device) for x in (src, rel, dst)]
    pos, rd, rs = tr.eval_scores(*d_ids)
    dev = lambda x: torch.from_numpy(x).to(tr.device)
    mar.mar_eval_filter(tr.ctx, d_ids[0], d_ids[1], d_ids[2], n, dev(doff), dev(dids), dev(soff), dev(sids), pos, rd, rs)
    torch.cuda.synchronize()
    got_d, got_s = rd.cpu().numpy(), rs.cpu().numpy()
    tr.close()
    ed, es = ostep.filtered_ranks(model, ne, re_, src, rel, dst, true_edges)
    ne64, re64 = ne.astype(np.float64), re_.astype(np.float64)
    sure = 0
    for e in range(n):
        s_, r_, d_ = int(src[e]), int(rel[e]), int(dst[e])
        p = float(models.score(model, ne64[s_], re64[r_], ne64[d_]))
        for got, exp, scores, own, listed in (
                (got_d[e], ed[e], models.score(model, ne64[s_][None, :], re64[r_][None, :], ne64), d_, dlist[e]),
                (got_s[e], es[e], models.score(model, ne64, re64[r_][None, :], ne64[d_][None, :]), s_, slist[e])):
            tol = 2e-6 * max(np.max(np.abs(scores)), abs(p))
            keep = np.ones(V, bool); keep[listed] = False
            # all nodes counted on the matrix cores (own endpoint included), listed candidates taken out on the vector ALU
            lo = 1 + np.sum(scores > p + tol) - np.sum(scores[listed] > p - tol)
            hi = 1 + np.sum(scores > p - tol) - np.sum(scores[listed] > p + tol)
            assert got >= 1 and max(lo, 1) <= got <= max(hi, 1), (e, got, lo, hi)
            near = np.abs(scores - p) <= tol
            near[own] = False
            if not near.any():
                # no other candidate near the edge's score: the rank is the oracle's, or one more if the matrix-core
                # score of the edge's own endpoint (a candidate like any other) rounds above the positive score
                assert int(got) - int(exp) in (0, 1), (e, got, exp)
                sure += 1
    print("filtered ranks decided without a margin:", sure, "of", 2 * n, flush=True)
    assert sure >= n // 4


def test_degree_based_evaluation_negatives_end_to_end():
    """Evaluation with a sampled candidate set of which a fraction is drawn by degree (Sec. 5.1, "Evaluation Task
    and Metrics": n_e negatives, alpha_ne of them by degree): mar_sample_negatives -> mar_eval_scores ->
    mar_rank_metrics against the oracle's sampler, ranks and metric reduction on the same seeded inputs."""
    from oracle import metrics, sampling
    import synth
    V, R, dim, B, C, N, Ndeg, seed, step = 3000, 6, 24, 600, 3, 400, 200, 9, 17
    rng = np.random.default_rng(5)
    ne = rng.integers(-2, 3, (V, dim)).astype(np.float32)           # small integers: every rank is exact
    re_ = rng.integers(-2, 3, (R, dim)).astype(np.float32)
    es, er, ed = (t.numpy() for t in synth.make_graph(V, R, 20000, 1.2, 1.0, seed=3))
    n = 530                                                         # a short last chunk
    src, rel, dst = es[:n].copy(), er[:n].copy(), ed[:n].copy()
    tr = mar.Trainer(V, R, dim, mar.MODEL_COMPLEX, B, C, N, Ndeg, seed=seed, node_emb=ne, rel_emb=re_)
    d_es, d_ed = torch.from_numpy(es).to(tr.device), torch.from_numpy(ed).to(tr.device)
    tr.sample_negatives(step, d_es, d_ed)
    pos, rd, rs = tr.eval_scores(*(torch.from_numpy(x).to(tr.device) for x in (src, rel, dst)))
    both = torch.cat([rd, rs]).contiguous()
    ks = [1, 10, 100]
    out = torch.zeros(1 + len(ks), dtype=torch.float64, device=tr.device)
    mar.mar_rank_metrics(tr.ctx, both, both.numel(), ks, out)
    torch.cuda.synchronize()
    nsrc, ndst = sampling.sample_negatives(seed, step, V, es, ed, C, N, Ndeg)
    assert np.array_equal(tr.neg_src.cpu().numpy().reshape(C, N), nsrc)
    assert np.array_equal(tr.neg_dst.cpu().numpy().reshape(C, N), ndst)
    # the degree-drawn slots follow the degree histogram: the hot nodes of the edge list show up far more often
    deg = np.bincount(ed, minlength=V)
    hot = np.argsort(-deg)[:30]
    assert np.isin(ndst[:, :Ndeg], hot).mean() > 5 * np.isin(ndst[:, Ndeg:], hot).mean()
    opos, ord_, ors = ostep.eval_scores(mar.MODEL_COMPLEX, B // C, ne, re_, src, rel, dst, nsrc, ndst)
    assert np.array_equal(pos.cpu().numpy(), opos.astype(np.float32))
    assert np.array_equal(rd.cpu().numpy(), ord_) and np.array_equal(rs.cpu().numpy(), ors)
    ranks = np.concatenate([ord_, ors])
    got = out.cpu().numpy()
    assert abs(got[0] - metrics.mrr(ranks)) <= 1e-12
    for j, k in enumerate(ks):
        assert got[1 + j] == metrics.hits_at(ranks, k)
    tr.close()
