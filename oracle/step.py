"""One synchronous training step and link-prediction scoring (oracle side; test
infrastructure).  Follows Alg. 1's body with all tables resident: form the batch,
compute gradients of Eq. 1's loss with sampled negatives (Sec. 2.1), update
relation and node parameters with Adagrad (Sec. 5.1).

Readings of points the paper leaves open (the same list is in the design notes):
* the batch is cut into contiguous chunks of ``chunk_size`` edges; chunk c has its
  own negative sets neg_src[c], neg_dst[c], shared by all its edges;
* both endpoints are corrupted, each with its own negative set; per edge
      L_e = -2 f(e) + log sum_j exp f(s_e, r_e, n_j) + log sum_j exp f(m_j, r_e, d_e)
  i.e. Eq. 1 applied once per corrupted side; the positive is not part of the
  log-sum (Eq. 1 as printed); no filtering of negatives that collide with the edge;
* the gradient is that of the SUM over the batch;
* Adagrad (Duchi et al.): state += G*G; theta -= lr * G / (sqrt(state) + eps),
  applied once per touched row per step with G summed over every occurrence of
  the row in the batch (as source, destination, relation or negative);
* tables are stored in fp32; the step is evaluated in fp64 from the fp32 values
  and rounded to fp32 once when stored back.
Ranks (Sec. 5.1, metrics): 1 + number of negatives scoring strictly higher.
"""
import numpy as np

from . import models

SIDE_SRC = models.SIDE_SRC
SIDE_DST = models.SIDE_DST


def _lse(x):
    m = np.max(x, axis=1, keepdims=True)
    return (m + np.log(np.sum(np.exp(x - m), axis=1, keepdims=True)))[:, 0]


class StepResult:
    """loss_sum: L summed over the batch; pos[n]; lse_dst[n] / lse_src[n]: the two
    log-sum terms per edge; uniq_nodes / uniq_rels: ascending unique touched ids;
    G_nodes[U, dim] / G_rels[Ur, dim]: summed gradients per unique row."""
    pass


def train_batch(model, lr, eps, chunk_size, node_emb, node_state, rel_emb, rel_state,
                src, rel, dst, neg_src, neg_dst, apply_update=True):
    src = np.asarray(src, dtype=np.int64)
    rel = np.asarray(rel, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    n = src.shape[0]
    dim = node_emb.shape[1]
    res = StepResult()
    if n == 0:
        res.loss_sum = 0.0
        res.pos = np.zeros(0); res.lse_dst = np.zeros(0); res.lse_src = np.zeros(0)
        res.uniq_nodes = np.zeros(0, dtype=np.int32); res.uniq_rels = np.zeros(0, dtype=np.int32)
        res.G_nodes = np.zeros((0, dim)); res.G_rels = np.zeros((0, dim))
        return res
    nchunks = (n + chunk_size - 1) // chunk_size
    neg_src = np.asarray(neg_src, dtype=np.int64)[:nchunks]
    neg_dst = np.asarray(neg_dst, dtype=np.int64)[:nchunks]

    uniq_nodes = np.unique(np.concatenate([src, dst, neg_src.ravel(), neg_dst.ravel()]))
    # Dot has no relation parameters: no relation row is touched
    uniq_rels = np.unique(rel) if model != models.DOT else np.zeros(0, dtype=np.int64)
    G_nodes = np.zeros((uniq_nodes.shape[0], dim), dtype=np.float64)
    G_rels = np.zeros((uniq_rels.shape[0], dim), dtype=np.float64)
    node_row = lambda ids: np.searchsorted(uniq_nodes, ids)
    rel_row = lambda ids: np.searchsorted(uniq_rels, ids)

    pos = np.empty(n); lse_dst = np.empty(n); lse_src = np.empty(n)
    for c in range(nchunks):
        lo, hi = c * chunk_size, min((c + 1) * chunk_size, n)
        s_id, r_id, d_id = src[lo:hi], rel[lo:hi], dst[lo:hi]
        S = node_emb[s_id].astype(np.float64)
        R = rel_emb[r_id].astype(np.float64)
        D = node_emb[d_id].astype(np.float64)

        # positive term: -2 f(e)
        pos[lo:hi] = models.score(model, S, R, D)
        fs, fr, fd = models.score_grads(model, S, R, D)
        np.add.at(G_nodes, node_row(s_id), -2.0 * fs)
        if model != models.DOT:
            np.add.at(G_rels, rel_row(r_id), -2.0 * fr)
        np.add.at(G_nodes, node_row(d_id), -2.0 * fd)

        # one log-sum-exp term per corrupted side
        for side, neg_ids, lse_out in ((SIDE_DST, neg_dst[c], lse_dst), (SIDE_SRC, neg_src[c], lse_src)):
            Neg = node_emb[neg_ids].astype(np.float64)
            A = models.neg_block(model, side, S, R, D, Neg)
            lse = _lse(A)
            lse_out[lo:hi] = lse
            P = np.exp(A - lse[:, None])                       # d lse_e / d A[e, j]
            gS, gR, gD, gNeg = models.neg_block_backward(model, side, S, R, D, Neg, P)
            np.add.at(G_nodes, node_row(s_id), gS)
            if model != models.DOT:
                np.add.at(G_rels, rel_row(r_id), gR)
            np.add.at(G_nodes, node_row(d_id), gD)
            np.add.at(G_nodes, node_row(neg_ids), gNeg)

    res.pos = pos; res.lse_dst = lse_dst; res.lse_src = lse_src
    res.loss_sum = float(np.sum(-2.0 * pos + lse_dst + lse_src))
    res.uniq_nodes = uniq_nodes.astype(np.int32)
    res.uniq_rels = uniq_rels.astype(np.int32)
    res.G_nodes = G_nodes
    res.G_rels = G_rels
    if apply_update:
        adagrad_rows(node_emb, node_state, uniq_nodes, G_nodes, lr, eps)
        adagrad_rows(rel_emb, rel_state, uniq_rels, G_rels, lr, eps)
    return res


def adagrad_rows(emb, state, rows, G, lr, eps):
    """Adagrad on the listed (unique) rows of fp32 tables, in place."""
    st = state[rows].astype(np.float64) + G * G
    th = emb[rows].astype(np.float64) - float(lr) * G / (np.sqrt(st) + float(eps))
    state[rows] = st.astype(np.float32)
    emb[rows] = th.astype(np.float32)


def eval_scores(model, chunk_size, node_emb, rel_emb, src, rel, dst, neg_src, neg_dst, return_blocks=False):
    """Positive scores and ranks against the chunk-shared negatives.
    Returns (pos[n], rank_dst[n], rank_src[n]) and, on request, the per-chunk score
    blocks [(A_dst, A_src), ...]."""
    src = np.asarray(src, dtype=np.int64)
    rel = np.asarray(rel, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    n = src.shape[0]
    nchunks = (n + chunk_size - 1) // chunk_size
    pos = np.empty(n)
    rank_dst = np.empty(n, dtype=np.int32)
    rank_src = np.empty(n, dtype=np.int32)
    blocks = []
    for c in range(nchunks):
        lo, hi = c * chunk_size, min((c + 1) * chunk_size, n)
        S = node_emb[src[lo:hi]].astype(np.float64)
        R = rel_emb[rel[lo:hi]].astype(np.float64)
        D = node_emb[dst[lo:hi]].astype(np.float64)
        pos[lo:hi] = models.score(model, S, R, D)
        A = models.neg_block(model, SIDE_DST, S, R, D, node_emb[np.asarray(neg_dst[c], dtype=np.int64)].astype(np.float64))
        Bm = models.neg_block(model, SIDE_SRC, S, R, D, node_emb[np.asarray(neg_src[c], dtype=np.int64)].astype(np.float64))
        rank_dst[lo:hi] = 1 + np.sum(A > pos[lo:hi, None], axis=1)
        rank_src[lo:hi] = 1 + np.sum(Bm > pos[lo:hi, None], axis=1)
        if return_blocks:
            blocks.append((A, Bm))
    if return_blocks:
        return pos, rank_dst, rank_src, blocks
    return pos, rank_dst, rank_src


def filtered_ranks(model, node_emb, rel_emb, src, rel, dst, true_edges):
    """Filtered link-prediction ranks (Sec. 5.1): every node is a candidate for the corrupted endpoint;
    candidates that make another TRUE edge (a false negative) are left out; rank = 1 + number of remaining
    candidates scoring strictly higher than the edge itself.  ``true_edges`` is an iterable of (s, r, d).
    Returns (rank_dst, rank_src).  Plain loops over edges: for small graphs only."""
    true_set = set((int(a), int(b), int(c)) for a, b, c in true_edges)
    ne = node_emb.astype(np.float64)
    re_ = rel_emb.astype(np.float64)
    V = ne.shape[0]
    n = len(src)
    rank_dst = np.empty(n, dtype=np.int32)
    rank_src = np.empty(n, dtype=np.int32)
    for e in range(n):
        s, r, d = int(src[e]), int(rel[e]), int(dst[e])
        pos = float(models.score(model, ne[s], re_[r], ne[d]))
        a = models.score(model, ne[s][None, :], re_[r][None, :], ne)            # all destinations
        keep = np.array([(c == d) or ((s, r, c) not in true_set) for c in range(V)])
        rank_dst[e] = 1 + int(np.sum((a > pos) & keep))
        b = models.score(model, ne, re_[r][None, :], ne[d][None, :])            # all sources
        keep = np.array([(c == s) or ((c, r, d) not in true_set) for c in range(V)])
        rank_src[e] = 1 + int(np.sum((b > pos) & keep))
    return rank_dst, rank_src
