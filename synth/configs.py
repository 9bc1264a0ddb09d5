"""The five synthetic workloads (sizes after Table 1 of the paper and Sec. 1's
400-dimensional / 50M-node example; skew parameters are this build's choice)."""
from dataclasses import dataclass, replace

DISTMULT, COMPLEX, TRANSE, DOT = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    num_nodes: int
    num_rels: int
    num_edges: int
    model: int
    dim: int
    batch_size: int
    num_chunks: int
    negs_per_chunk: int
    deg_negs_per_chunk: int
    node_zipf: float          # exponent of the node popularity law (src and dst drawn independently)
    rel_zipf: float           # 0 -> uniform relations
    lr: float = 0.1
    eps: float = 1e-10
    init_std: float = 0.001
    seed: int = 0

    @property
    def chunk_size(self):
        return self.batch_size // self.num_chunks

    def scaled(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    # 1: tiny graph, one epoch = 100 steps
    "tiny": Workload("tiny", 10_000, 10, 100_000, DISTMULT, 50, 1_000, 10, 100, 0, 1.1, 0.0),
    # 2: shape of a small knowledge graph (|V| ~ 15k, |R| ~ 1.3k), the benchmark workload
    "kg_small": Workload("kg_small", 14_951, 1_345, 483_142, COMPLEX, 100, 10_000, 10, 1_000, 100, 1.2, 1.0),
    # 3: shape of a large social graph, single relation
    "social": Workload("social", 41_600_000, 1, 1_460_000_000, DISTMULT, 100, 50_000, 50, 1_000, 0, 1.8, 0.0),
    # 3b: the same graph with the relation-free Dot score the paper trains social graphs with (Sec. 5.1)
    "social_dot": Workload("social_dot", 41_600_000, 1, 1_460_000_000, DOT, 100, 50_000, 50, 1_000, 0, 1.8, 0.0),
    # 4: shape of a large knowledge graph
    "kg_large": Workload("kg_large", 86_100_000, 14_824, 338_000_000, COMPLEX, 100, 50_000, 50, 1_000, 500, 1.3, 1.3),
    # 5: wide embeddings, 80 GB table + 80 GB optimiser state
    "wide": Workload("wide", 50_000_000, 1_000, 500_000_000, DISTMULT, 400, 100_000, 100, 1_000, 0, 1.2, 0.0),
}


def get_workload(name):
    return CONFIGS[name]
