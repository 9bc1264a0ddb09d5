"""Training with bounded staleness (oracle side; test infrastructure).

Sec. 3 of the paper: node embeddings (and their optimiser state) live in CPU memory and move through a
pipeline -- gather and transfer to the GPU, compute, transfer the node gradients back, apply them on the CPU --
of which up to a fixed number of batches are in flight at once; relation embeddings stay on the GPU and are
updated synchronously ("Bounded Staleness": only node embeddings are read stale).  With ``staleness`` = s the
node rows batch j reads are the ones in CPU memory after the node updates of batches 0 .. j-1-s have been
applied, and nothing later; batch j's own node gradient, computed from those rows and the CURRENT relation
rows, is applied to whatever the CPU copy holds when its turn comes (updates are applied in batch order; Stage 5:
the scaled gradient is added to the current version).  s = 0 is the synchronous loop of Alg. 1.

The optimiser is Adagrad as in step.py, so "applying" batch j's node gradient G means, on the current CPU rows,
state += G*G; theta -= lr * G / (sqrt(state) + eps).
"""
import numpy as np

from . import step as ostep


def train_pipelined(model, lr, eps, chunk_size, node_emb, node_state, rel_emb, rel_state, batches, staleness):
    """``batches``: iterable of (src, rel, dst, neg_src, neg_dst).  Tables are updated in place.
    Returns the list of per-batch loss sums."""
    pending = []                       # node updates computed but not yet applied: (unique node ids, G), oldest first
    losses = []
    for src, rel, dst, neg_src, neg_dst in batches:
        # the CPU copy batch j reads holds the node updates of batches <= j-1-s
        while len(pending) > staleness:
            rows, G = pending.pop(0)
            ostep.adagrad_rows(node_emb, node_state, rows, G, lr, eps)
        # gradients from the (possibly stale) node rows and the current relation rows; no table is touched
        res = ostep.train_batch(model, lr, eps, chunk_size, node_emb, node_state, rel_emb, rel_state,
                                src, rel, dst, neg_src, neg_dst, apply_update=False)
        losses.append(res.loss_sum)
        ostep.adagrad_rows(rel_emb, rel_state, res.uniq_rels.astype(np.int64), res.G_rels, lr, eps)   # relations: synchronous
        pending.append((res.uniq_nodes.astype(np.int64), res.G_nodes))
    for rows, G in pending:
        ostep.adagrad_rows(node_emb, node_state, rows, G, lr, eps)
    return losses
