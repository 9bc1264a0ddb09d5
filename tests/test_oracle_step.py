"""Pins for the oracle's training step: brute-force loops, finite differences of
the whole loss, torch.autograd on a dense restatement, loss closed forms, Adagrad
invariants and library routine, rank brute force."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import models, step
from oracle.models import DISTMULT, COMPLEX, TRANSE, DOT

ALL = (DISTMULT, COMPLEX, TRANSE, DOT)


def tiny(seed, V=12, Rn=3, dim=6, n=7, S=4, N=3, scale=0.7):
    rng = np.random.default_rng(seed)
    C = (n + S - 1) // S
    t = dict(
        node_emb=(rng.standard_normal((V, dim)) * scale).astype(np.float32),
        rel_emb=(rng.standard_normal((Rn, dim)) * scale).astype(np.float32),
        src=rng.integers(0, V, n), rel=rng.integers(0, Rn, n), dst=rng.integers(0, V, n),
        neg_src=rng.integers(0, V, (C, N)), neg_dst=rng.integers(0, V, (C, N)), S=S)
    t["node_state"] = np.zeros_like(t["node_emb"]); t["rel_state"] = np.zeros_like(t["rel_emb"])
    return t


def run(model, t, lr=0.1, eps=1e-10, apply_update=True):
    return step.train_batch(model, lr, eps, t["S"], t["node_emb"], t["node_state"], t["rel_emb"], t["rel_state"],
                            t["src"], t["rel"], t["dst"], t["neg_src"], t["neg_dst"], apply_update=apply_update)


def loop_loss(model, node_emb, rel_emb, t):
    """Eq. 1 with sampled negatives, one edge and one negative at a time."""
    L = 0.0
    for e in range(len(t["src"])):
        c = e // t["S"]
        s, r, d = node_emb[t["src"][e]], rel_emb[t["rel"][e]], node_emb[t["dst"][e]]
        f = float(models.score(model, s, r, d))
        za = sum(math.exp(float(models.score(model, s, r, node_emb[j]))) for j in t["neg_dst"][c])
        zb = sum(math.exp(float(models.score(model, node_emb[j], r, d))) for j in t["neg_src"][c])
        L += -(f - math.log(za)) - (f - math.log(zb))
    return L


@pytest.mark.parametrize("model", ALL)
def test_loss_equals_edge_by_edge_loop(model):
    t = tiny(model)
    res = run(model, t, apply_update=False)
    ref = loop_loss(model, t["node_emb"].astype(np.float64), t["rel_emb"].astype(np.float64), t)
    assert np.isclose(res.loss_sum, ref, rtol=1e-12)
    assert np.isclose(res.loss_sum, np.sum(-2 * res.pos + res.lse_dst + res.lse_src), rtol=1e-14)


@pytest.mark.parametrize("model", ALL)
def test_gradients_by_central_differences_of_the_loop_loss(model):
    t = tiny(10 + model, V=9, Rn=2, dim=4, n=6, S=3, N=3)
    res = run(model, t, apply_update=False)
    ne = t["node_emb"].astype(np.float64); re_ = t["rel_emb"].astype(np.float64)
    h = 1e-6
    Gn = np.zeros_like(ne); Gr = np.zeros_like(re_)
    for tab, G in ((ne, Gn), (re_, Gr)):
        for i in range(tab.shape[0]):
            for k in range(tab.shape[1]):
                old = tab[i, k]
                tab[i, k] = old + h; fp = loop_loss(model, ne, re_, t)
                tab[i, k] = old - h; fm = loop_loss(model, ne, re_, t)
                tab[i, k] = old
                G[i, k] = (fp - fm) / (2 * h)
    assert np.allclose(Gn[res.uniq_nodes], res.G_nodes, atol=5e-7)
    assert np.allclose(Gr[res.uniq_rels], res.G_rels, atol=5e-7)
    untouched = np.setdiff1d(np.arange(ne.shape[0]), res.uniq_nodes)
    assert np.all(np.abs(Gn[untouched]) < 1e-9)


def _torch_loss(model, ne, re_, t):
    def f(s, r, d):
        if model == DISTMULT:
            return (s * r * d).sum(-1)
        if model == COMPLEX:
            h = s.shape[-1] // 2
            sr, si, rr, ri, dr, di = s[..., :h], s[..., h:], r[..., :h], r[..., h:], d[..., :h], d[..., h:]
            return (sr * rr * dr + si * rr * di + sr * ri * di - si * ri * dr).sum(-1)
        if model == DOT:
            return (s * d).sum(-1) + 0.0 * r.sum(-1)
        return -torch.linalg.vector_norm(s + r - d, dim=-1)
    L = 0.0
    n = len(t["src"])
    for c in range((n + t["S"] - 1) // t["S"]):
        lo, hi = c * t["S"], min((c + 1) * t["S"], n)
        s = ne[torch.as_tensor(t["src"][lo:hi])]; r = re_[torch.as_tensor(t["rel"][lo:hi])]
        d = ne[torch.as_tensor(t["dst"][lo:hi])]
        nd = ne[torch.as_tensor(t["neg_dst"][c])]; ns = ne[torch.as_tensor(t["neg_src"][c])]
        pos = f(s, r, d)
        a = f(s[:, None, :], r[:, None, :], nd[None, :, :])
        b = f(ns[None, :, :], r[:, None, :], d[:, None, :])
        L = L + (-2 * pos + torch.logsumexp(a, 1) + torch.logsumexp(b, 1)).sum()
    return L


@pytest.mark.parametrize("model", ALL)
def test_gradients_against_torch_autograd(model):
    t = tiny(20 + model, V=40, Rn=5, dim=8, n=23, S=8, N=6)
    res = run(model, t, apply_update=False)
    ne = torch.tensor(t["node_emb"], dtype=torch.float64, requires_grad=True)
    re_ = torch.tensor(t["rel_emb"], dtype=torch.float64, requires_grad=True)
    L = _torch_loss(model, ne, re_, t)
    L.backward()
    assert np.isclose(L.item(), res.loss_sum, rtol=1e-12)
    assert np.allclose(ne.grad.numpy()[res.uniq_nodes], res.G_nodes, rtol=1e-9, atol=1e-12)
    assert np.allclose(re_.grad.numpy()[res.uniq_rels], res.G_rels, rtol=1e-9, atol=1e-12)
    mask = np.ones(40, bool); mask[res.uniq_nodes] = False
    assert np.all(ne.grad.numpy()[mask] == 0)


def test_unique_sets_and_partial_batch():
    t = tiny(5, n=7, S=4, N=3)                     # two chunks, the second has 3 edges
    res = run(DISTMULT, t, apply_update=False)
    ids = np.concatenate([t["src"], t["dst"], t["neg_src"].ravel(), t["neg_dst"].ravel()])
    assert np.array_equal(res.uniq_nodes, np.unique(ids))
    assert np.all(np.diff(res.uniq_nodes) > 0)
    assert np.array_equal(res.uniq_rels, np.unique(t["rel"]))
    # negatives of chunks beyond the batch's last edge are not used
    t2 = dict(t); t2["src"], t2["rel"], t2["dst"] = t["src"][:3], t["rel"][:3], t["dst"][:3]
    r2 = run(DISTMULT, t2, apply_update=False)
    ids2 = np.concatenate([t2["src"], t2["dst"], t["neg_src"][0], t["neg_dst"][0]])
    assert np.array_equal(r2.uniq_nodes, np.unique(ids2))
    r0 = step.train_batch(DISTMULT, 0.1, 1e-10, 4, t["node_emb"], t["node_state"], t["rel_emb"], t["rel_state"],
                          [], [], [], t["neg_src"], t["neg_dst"])
    assert r0.loss_sum == 0.0 and r0.uniq_nodes.size == 0


def test_loss_closed_forms():
    # N = 1: each side term is a - pos
    t = tiny(7, n=5, S=5, N=1)
    res = run(DISTMULT, t, apply_update=False)
    ne, re_ = t["node_emb"].astype(np.float64), t["rel_emb"].astype(np.float64)
    a = models.score(DISTMULT, ne[t["src"]], re_[t["rel"]], ne[t["neg_dst"][0, 0]][None, :])
    b = models.score(DISTMULT, ne[t["neg_src"][0, 0]][None, :], re_[t["rel"]], ne[t["dst"]])
    assert np.allclose(res.lse_dst, a) and np.allclose(res.lse_src, b)
    assert np.isclose(res.loss_sum, np.sum(a + b - 2 * res.pos))
    # all tables zero: every score is 0, each side term is log N
    t = tiny(8, n=6, S=3, N=5)
    t["node_emb"][:] = 0
    res = run(DISTMULT, t, apply_update=False)
    assert np.isclose(res.loss_sum, 6 * 2 * math.log(5))
    # library log-sum-exp, and shift invariance
    x = np.random.default_rng(0).standard_normal((4, 9)) * 30
    assert np.allclose(step._lse(x), logsumexp(x, axis=1), rtol=1e-14)
    assert np.allclose(step._lse(x + 1000.0), step._lse(x) + 1000.0, rtol=1e-14)
    assert np.all(np.isfinite(step._lse(x * 40)))
    # loss at N(0, 0.001^2) initialisation is about 2 log N per edge
    t = tiny(9, V=500, Rn=4, dim=50, n=200, S=100, N=100, scale=0.001)
    res = run(DISTMULT, t, apply_update=False)
    assert abs(res.loss_sum / 200 - 2 * math.log(100)) < 1e-4


@pytest.mark.parametrize("model", ALL)
def test_softmax_weights_sum_to_one(model):
    # d(lse_e)/d(a_e.) sums to 1: scaling identity for scores linear in the negative
    # is model specific, so check through the block directly
    t = tiny(30 + model)
    ne = t["node_emb"].astype(np.float64); re_ = t["rel_emb"].astype(np.float64)
    S, R, D = ne[t["src"][:4]], re_[t["rel"][:4]], ne[t["dst"][:4]]
    A = models.neg_block(model, models.SIDE_DST, S, R, D, ne[t["neg_dst"][0]])
    P = np.exp(A - step._lse(A)[:, None])
    assert np.allclose(P.sum(1), 1.0, rtol=1e-13)


@pytest.mark.parametrize("model", ALL)
def test_adagrad_invariants(model):
    t = tiny(40 + model, V=30)
    ne0, re0 = t["node_emb"].copy(), t["rel_emb"].copy()
    res = run(model, t)
    touched = np.zeros(30, bool); touched[res.uniq_nodes] = True
    assert np.array_equal(t["node_emb"][~touched], ne0[~touched])          # untouched rows bit-identical
    assert np.all(t["node_state"][~touched] == 0)
    assert (~touched).sum() > 0
    # first step from zero state: lr * G / (|G| + eps)
    G = res.G_nodes
    exp = ne0[res.uniq_nodes].astype(np.float64) - 0.1 * G / (np.abs(G) + 1e-10)
    assert np.array_equal(t["node_emb"][res.uniq_nodes], exp.astype(np.float32))
    assert np.array_equal(t["node_state"][res.uniq_nodes], (G * G).astype(np.float32))
    # second step: state never decreases
    st1n, st1r = t["node_state"].copy(), t["rel_state"].copy()
    run(model, t)
    assert np.all(t["node_state"] >= st1n) and np.all(t["rel_state"] >= st1r)
    assert np.any(t["node_state"] > st1n)


def test_adagrad_matches_library_on_summed_sparse_gradient():
    t = tiny(50, V=15, Rn=3, dim=5, n=9, S=3, N=4)
    ne = torch.tensor(t["node_emb"], dtype=torch.float64, requires_grad=True)
    re_ = torch.tensor(t["rel_emb"], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adagrad([ne, re_], lr=0.1, eps=1e-10, initial_accumulator_value=0.0)
    ref = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in t.items()}
    for _ in range(3):
        opt.zero_grad()
        _torch_loss(DISTMULT, ne, re_, t).backward()
        opt.step()
        run(DISTMULT, ref)
        # the oracle stores fp32 between steps; keep the library on the same values
        with torch.no_grad():
            assert np.allclose(ne.numpy(), ref["node_emb"], rtol=2e-7, atol=1e-9)
            assert np.allclose(re_.numpy(), ref["rel_emb"], rtol=2e-7, atol=1e-9)
            ne.copy_(torch.tensor(ref["node_emb"], dtype=torch.float64))
            re_.copy_(torch.tensor(ref["rel_emb"], dtype=torch.float64))
            opt.state[ne]["sum"].copy_(torch.tensor(ref["node_state"], dtype=torch.float64))
            opt.state[re_]["sum"].copy_(torch.tensor(ref["rel_state"], dtype=torch.float64))


def test_duplicate_occurrences_get_one_update_with_the_summed_gradient():
    t = tiny(60, n=4, S=4, N=3)
    # duplicate edge 0 as edge 1: G of the batch = G of the batch with one copy, plus that edge's terms again
    for k in ("src", "rel", "dst"):
        t[k][1] = t[k][0]
    res = run(DISTMULT, t, apply_update=False)
    one = dict(t); sel = [0, 2, 3]
    for k in ("src", "rel", "dst"):
        one[k] = t[k][sel]
    r_one = run(DISTMULT, one, apply_update=False)
    only = dict(t)
    for k in ("src", "rel", "dst"):
        only[k] = t[k][[0]]
    r_only = run(DISTMULT, only, apply_update=False)
    G = np.zeros((12, 6)); G[r_one.uniq_nodes] += r_one.G_nodes; G[r_only.uniq_nodes] += r_only.G_nodes
    assert np.allclose(G[res.uniq_nodes], res.G_nodes, rtol=1e-12, atol=1e-15)
    # and the update is a single Adagrad step with that sum (not two steps)
    before = t["node_emb"].copy()
    res = run(DISTMULT, t)
    row = t["src"][0]
    g = res.G_nodes[np.searchsorted(res.uniq_nodes, row)]
    assert np.array_equal(t["node_emb"][row], (before[row].astype(np.float64) - 0.1 * g / (np.abs(g) + 1e-10)).astype(np.float32))


@pytest.mark.parametrize("model", ALL)
def test_ranks_by_brute_force_sort(model):
    t = tiny(70 + model, V=25, n=11, S=4, N=6)
    # small-integer embeddings: every score is exact in fp64 whatever the summation order, so
    # ties (a negative that is the edge's own endpoint) are exact and rank optimistically
    rng = np.random.default_rng(model)
    t["node_emb"] = rng.integers(-3, 4, t["node_emb"].shape).astype(np.float32)
    t["rel_emb"] = rng.integers(-3, 4, t["rel_emb"].shape).astype(np.float32)
    t["neg_dst"][0, 0] = t["dst"][1]                     # a guaranteed tie
    pos, rd, rs, blocks = step.eval_scores(model, t["S"], t["node_emb"], t["rel_emb"], t["src"], t["rel"], t["dst"],
                                           t["neg_src"], t["neg_dst"], return_blocks=True)
    ne = t["node_emb"].astype(np.float64); re_ = t["rel_emb"].astype(np.float64)
    for e in range(11):
        c = e // 4
        f = float(models.score(model, ne[t["src"][e]], re_[t["rel"][e]], ne[t["dst"][e]]))
        assert np.isclose(pos[e], f)
        for ranks, neg in ((rd, [float(models.score(model, ne[t["src"][e]], re_[t["rel"][e]], ne[j])) for j in t["neg_dst"][c]]),
                           (rs, [float(models.score(model, ne[j], re_[t["rel"][e]], ne[t["dst"][e]])) for j in t["neg_src"][c]])):
            order = sorted(neg + [f], reverse=True)           # position in the descending array, first match
            assert ranks[e] == order.index(f) + 1
            assert 1 <= ranks[e] <= 7
    assert len(blocks) == 3 and blocks[2][0].shape == (3, 6)


def test_training_reduces_the_loss():
    t = tiny(80, V=60, Rn=3, dim=8, n=40, S=10, N=8, scale=0.1)
    losses = [run(DISTMULT, t).loss_sum for _ in range(15)]
    assert losses[-1] < losses[0] - 1.0


def test_filtered_ranks_properties_and_brute_force():
    rng = np.random.default_rng(5)
    V, Rn, dim = 15, 2, 4
    ne = rng.integers(-3, 4, (V, dim)).astype(np.float32)            # exact arithmetic, ties included
    re_ = rng.integers(-3, 4, (Rn, dim)).astype(np.float32)
    edges = [(int(rng.integers(V)), int(rng.integers(Rn)), int(rng.integers(V))) for _ in range(40)]
    src, rel, dst = (np.array(x) for x in zip(*edges[:12]))
    fd, fs = step.filtered_ranks(DISTMULT, ne, re_, src, rel, dst, edges)
    # unfiltered ranks against all nodes: every node once as a negative
    allnodes = np.arange(V)[None, :]
    _, ud, us = step.eval_scores(DISTMULT, 12, ne, re_, src, rel, dst, allnodes, allnodes)
    assert np.all(fd <= ud) and np.all(fs <= us) and np.all(fd >= 1) and np.all(fs >= 1)
    # with no other true edges nothing is filtered
    fd0, fs0 = step.filtered_ranks(DISTMULT, ne, re_, src, rel, dst, list(zip(src, rel, dst)))
    ok = [e for e in range(12) if sum(1 for t in zip(src, rel, dst) if t[0] == src[e] and t[1] == rel[e]) == 1]
    assert all(fd0[e] == ud[e] for e in ok)
    # brute force for one edge, one candidate at a time
    e = 3
    s, r, d = edges[e]
    f = lambda a, b, c: float(models.score(DISTMULT, ne[a].astype(float), re_[b].astype(float), ne[c].astype(float)))
    cnt = sum(1 for c in range(V) if (c == d or (s, r, c) not in set(edges)) and f(s, r, c) > f(s, r, d))
    assert fd[e] == 1 + cnt
    # filtering a candidate that outranks the edge lowers the rank by exactly one
    better = [c for c in range(V) if c != d and (s, r, c) not in set(edges) and f(s, r, c) > f(s, r, d)]
    if better:
        fd2, _ = step.filtered_ranks(DISTMULT, ne, re_, src[e:e + 1], rel[e:e + 1], dst[e:e + 1], edges + [(s, r, better[0])])
        assert fd2[0] == fd[e] - 1
