"""GPU parity over many steps: sampling + training through the C ABI against the oracle, mean loss
within rel 1e-3 after 100 steps (the stated bar), on the two workloads small enough to run whole."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar
import synth
from oracle import sampling, step as ostep

pytestmark = pytest.mark.gpu


def _train_both(w, steps, precision=0):
    src, rel, dst = synth.make_graph(w.num_nodes, w.num_rels, w.num_edges, w.node_zipf, w.rel_zipf, seed=w.seed)
    es, er, ed = src.numpy(), rel.numpy(), dst.numpy()
    ne = sampling.init_table(w.seed, 0, w.num_nodes, w.dim, np.float32(w.init_std)).astype(np.float32)
    re_ = sampling.init_table(w.seed, 1, w.num_rels, w.dim, np.float32(w.init_std)).astype(np.float32)
    tr = mar.Trainer(w.num_nodes, w.num_rels, w.dim, w.model, w.batch_size, w.num_chunks, w.negs_per_chunk,
                     w.deg_negs_per_chunk, w.lr, w.eps, w.init_std, w.seed, node_emb=ne, rel_emb=re_, precision=precision)
    d_src, d_rel, d_dst = src.to(tr.device), rel.to(tr.device), dst.to(tr.device)
    nb = (w.num_edges + w.batch_size - 1) // w.batch_size
    gpu_losses = torch.zeros(steps, device=tr.device)
    counts = []
    for i in range(steps):
        b = i % nb
        lo, hi = b * w.batch_size, min((b + 1) * w.batch_size, w.num_edges)
        tr.sample_negatives(i, d_src, d_dst)
        tr.train_batch(d_src[lo:hi], d_rel[lo:hi], d_dst[lo:hi])
        gpu_losses[i] = tr.loss[0]
        counts.append(hi - lo)
    torch.cuda.synchronize()
    gpu_losses = gpu_losses.cpu().numpy().astype(np.float64)
    gpu_tables = tr.node_emb.cpu().numpy(), tr.rel_emb.cpu().numpy()
    tr.close()

    ns, rs = np.zeros_like(ne), np.zeros_like(re_)
    ora_losses = []
    for i in range(steps):
        b = i % nb
        lo, hi = b * w.batch_size, min((b + 1) * w.batch_size, w.num_edges)
        nsrc, ndst = sampling.sample_negatives(w.seed, i, w.num_nodes, es, ed, w.num_chunks, w.negs_per_chunk,
                                               w.deg_negs_per_chunk)
        r = ostep.train_batch(w.model, np.float32(w.lr), np.float32(w.eps), w.chunk_size, ne, ns, re_, rs,
                              es[lo:hi], er[lo:hi], ed[lo:hi], nsrc, ndst)
        ora_losses.append(r.loss_sum)
        if i % 10 == 0:
            print("oracle step", i, r.loss_sum / (hi - lo), flush=True)
    return gpu_losses, np.array(ora_losses), np.array(counts, dtype=np.float64), gpu_tables, (ne, re_)


@pytest.mark.parametrize("precision", (0, 1))
@pytest.mark.parametrize("name,steps", (("tiny", 100), ("kg_small", 100)))
def test_mean_loss_after_100_steps(name, steps, precision):
    """precision 1: the split-precision contraction (bf16 hi + lo operands), held to the same bars."""
    w = synth.get_workload(name)
    g, o, cnt, gt, ot = _train_both(w, steps, precision)
    mean_g, mean_o = g / cnt, o / cnt
    # at initialisation every score is ~0: loss per edge = 2 log N
    assert abs(mean_o[0] - 2 * np.log(w.negs_per_chunk)) < 1e-3
    assert mean_o[-1] < mean_o[0]
    rel_final = abs(mean_g[-1] - mean_o[-1]) / abs(mean_o[-1])
    rel_run = abs(mean_g.mean() - mean_o.mean()) / abs(mean_o.mean())
    print(name, "final mean loss gpu/oracle", mean_g[-1], mean_o[-1], "rel", rel_final, "run-mean rel", rel_run, flush=True)
    assert rel_final <= 1e-3 and rel_run <= 1e-3
    # every step, not just the last.  The per-edge loss starts near 2 log N and, on the tiny graph, passes
    # through zero on its way down; there the bar is absolute (1e-3 of one loss unit) instead of relative to
    # the vanishing value.
    assert np.max(np.abs(mean_g - mean_o) / np.maximum(np.abs(mean_o), 1.0)) <= 1e-3
    # the trained tables themselves.  From a zero accumulator an element's first update is lr * sign(G), so an
    # element whose gradient is zero up to rounding can start +-2 lr apart in fp32 and fp64 and carries that
    # offset along; such elements are counted and bounded, all others must agree to 1e-3 of the table's scale.
    for tg, to in zip(gt, ot):
        scale = float(np.max(np.abs(to)))
        diff = np.abs(tg.astype(np.float64) - to.astype(np.float64))
        off = diff > 1e-3 * scale
        print(name, "table elements off by more than 1e-3 of scale:", int(off.sum()), "of", off.size,
              "largest", float(diff.max()) / scale, flush=True)
        # The number of such elements is proportional to the rounding level of the gradients (2^-24 relative in
        # fp32, about 2^-17 in split precision: 128 times more); observed fractions 0 .. 4e-5 in fp32 and
        # 9e-4 .. 5.5e-3 in split precision on these workloads.
        assert off.mean() <= (1e-4 if precision == 0 else 1e-2)
