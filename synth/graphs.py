"""Seeded edge-list generator (torch, any device).

Recipe: a node's popularity rank k in [1, V] is drawn with P(k) ~ k^-a by the
inverse CDF of the continuous power law on [1, V+1) and floored; ranks map to ids
through a fixed seeded permutation so hot rows are scattered over the table;
sources and destinations are drawn independently (out- and in-degree both follow
the law); relation ids are uniform (a = 0) or follow their own power law through
their own permutation.  Self loops and duplicate edges are allowed.  Edges come
out in random order, as int32 arrays.
"""
import torch


def _powerlaw_ranks(n, size, a, gen, device):
    """Zero-based popularity ranks in [0, size) with P(k) ~ (k+1)^-a."""
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float64)
    if a == 0.0:
        k = torch.floor(u * size)
    elif abs(a - 1.0) < 1e-12:
        k = torch.floor(torch.exp(u * torch.log(torch.tensor(float(size + 1), dtype=torch.float64)))) - 1
    else:
        top = float(size + 1) ** (1.0 - a)
        k = torch.floor(((top - 1.0) * u + 1.0) ** (1.0 / (1.0 - a))) - 1
    return k.clamp_(0, size - 1).to(torch.int64)


def zipf_ids(n, size, a, perm, gen, device):
    ranks = _powerlaw_ranks(n, size, a, gen, device)
    return perm[ranks] if perm is not None else ranks


def make_graph(num_nodes, num_rels, num_edges, node_zipf, rel_zipf, seed=0, device="cpu", block=1 << 26):
    """Returns (src, rel, dst) int32 tensors of length num_edges on ``device``."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    node_perm = torch.randperm(num_nodes, generator=gen, device=device)
    rel_perm = torch.randperm(num_rels, generator=gen, device=device) if rel_zipf != 0.0 else None
    src = torch.empty(num_edges, dtype=torch.int32, device=device)
    rel = torch.empty(num_edges, dtype=torch.int32, device=device)
    dst = torch.empty(num_edges, dtype=torch.int32, device=device)
    for lo in range(0, num_edges, block):
        hi = min(lo + block, num_edges)
        m = hi - lo
        src[lo:hi] = zipf_ids(m, num_nodes, node_zipf, node_perm, gen, device).to(torch.int32)
        dst[lo:hi] = zipf_ids(m, num_nodes, node_zipf, node_perm, gen, device).to(torch.int32)
        if num_rels == 1:
            rel[lo:hi] = 0
        else:
            rel[lo:hi] = zipf_ids(m, num_rels, rel_zipf, rel_perm, gen, device).to(torch.int32)
    return src, rel, dst


def make_tables(num_nodes, num_rels, dim, std, seed=0, device="cpu"):
    """Seeded N(0, std^2) node and relation tables (fp32) on ``device``: plain input data for runs whose
    tables are too large to build on the host."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) + 0x7AB1E5)
    node = torch.randn((num_nodes, dim), generator=gen, device=device, dtype=torch.float32).mul_(std)
    rel = torch.randn((num_rels, dim), generator=gen, device=device, dtype=torch.float32).mul_(std)
    return node, rel
