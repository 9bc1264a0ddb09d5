"""Negative sampling and table initialisation (oracle side; test infrastructure).

Sec. 2.1 approximates the log-term of Eq. 1 by a "(typically uniform) sample of
nodes"; Sec. 5.1 / Table 1 add a fraction alpha of negatives drawn by degree.
The paper gives no generator and no chunk structure; the reading taken is:

* one 64-bit random word per (seed, step, side, chunk, slot), taken from
  Philox4x32-10 with
      key     = (seed & 0xffffffff, seed >> 32)
      counter = (slot >> 1, 2*chunk + side, step & 0xffffffff, step >> 32)
  the block's output words (o0, o1, o2, o3) give x = o0 | o1 << 32 for even
  slots and x = o2 | o3 << 32 for odd slots; side 0 = negatives that replace the
  source, side 1 = negatives that replace the destination; step < 2**63;
* the first ``deg_negs`` slots of every chunk are degree-proportional: the id is
  the matching endpoint of edge number mulhi64(x, num_edges) (source endpoint for
  side 0, destination endpoint for side 1), i.e. proportional to out- / in-degree;
* the remaining slots are uniform node ids mulhi64(x, num_nodes).

Table initialisation N(0, std^2) uses the same generator in a disjoint counter
range (counter word 3 has its top bit set, which no sampling step reaches):
      counter = (block & 0xffffffff, block >> 32, 0, 0x80000000 | table)
for elements 4*block .. 4*block+3 of the flattened table (table 0 = node
embeddings, 1 = relation embeddings); with 24-bit uniforms
      u1 = ((o0 >> 8) + 1) / 2**24 in (0, 1],   u2 = (o1 >> 8) / 2**24 in [0, 1)
the Box-Muller pair is  sqrt(-2 ln u1) * (cos, sin)(2 pi u2); words o2, o3 give the
second pair.  Optimiser state starts at zero.
"""
import numpy as np

from .philox import philox4x32_10_np, mulhi64_np

SIDE_SRC = 0
SIDE_DST = 1


def random_words(seed, step, side, num_chunks, num_slots):
    """64-bit words x[chunk, slot] for one side of one step (uint64 array)."""
    seed = int(seed)
    step = int(step)
    assert 0 <= step < (1 << 63)
    slots = np.arange(num_slots, dtype=np.uint64)
    chunks = np.arange(num_chunks, dtype=np.uint64)
    c0 = (slots >> np.uint64(1))[None, :]
    c1 = (chunks * np.uint64(2) + np.uint64(side))[:, None]
    c2 = np.uint64(step & 0xFFFFFFFF)
    c3 = np.uint64(step >> 32)
    o0, o1, o2, o3 = philox4x32_10_np(c0, c1, c2, c3, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    even = o0 | (o1 << np.uint64(32))
    odd = o2 | (o3 << np.uint64(32))
    return np.where((slots & np.uint64(1))[None, :] == 0, even, odd)


def sample_negatives(seed, step, num_nodes, edge_src, edge_dst, num_chunks, negs_per_chunk, deg_negs):
    """Returns (neg_src[C, N], neg_dst[C, N]) int32: per chunk the ids that replace
    the source, and those that replace the destination."""
    edge_src = np.asarray(edge_src)
    edge_dst = np.asarray(edge_dst)
    num_edges = int(edge_src.shape[0])
    out = []
    for side, endpoints in ((SIDE_SRC, edge_src), (SIDE_DST, edge_dst)):
        x = random_words(seed, step, side, num_chunks, negs_per_chunk)
        ids = mulhi64_np(x, num_nodes).astype(np.int64)
        if deg_negs > 0:
            assert num_edges > 0
            eidx = mulhi64_np(x[:, :deg_negs], num_edges).astype(np.int64)
            ids[:, :deg_negs] = endpoints[eidx]
        out.append(ids.astype(np.int32))
    return out[0], out[1]


def init_table(seed, table, num_rows, dim, std):
    """fp64 values of the N(0, std^2) initialisation of one table, shape (num_rows, dim)."""
    seed = int(seed)
    n = int(num_rows) * int(dim)
    nblocks = (n + 3) // 4
    blk = np.arange(nblocks, dtype=np.uint64)
    o = philox4x32_10_np(blk & np.uint64(0xFFFFFFFF), blk >> np.uint64(32), np.uint64(0),
                         np.uint64(0x80000000 | int(table)), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    z = np.empty((nblocks, 4), dtype=np.float64)
    for pair in range(2):
        u1 = ((o[2 * pair] >> np.uint64(8)).astype(np.float64) + 1.0) / 16777216.0
        u2 = (o[2 * pair + 1] >> np.uint64(8)).astype(np.float64) / 16777216.0
        r = np.sqrt(-2.0 * np.log(u1))
        z[:, 2 * pair] = r * np.cos(2.0 * np.pi * u2)
        z[:, 2 * pair + 1] = r * np.sin(2.0 * np.pi * u2)
    return (z.reshape(-1)[:n] * float(std)).reshape(int(num_rows), int(dim))
