"""Link-prediction metrics from ranks (oracle side; test infrastructure).

Sec. 5.1, "Evaluation Task and Metrics": for candidate edges C with ranks r_i,
MRR = (1/|C|) sum_i 1/r_i and Hits@k = (1/|C|) sum_i [r_i <= k].
"""
import numpy as np


def mrr(ranks):
    ranks = np.asarray(ranks, dtype=np.float64)
    return float(np.sum(1.0 / ranks) / ranks.size) if ranks.size else 0.0


def hits_at(ranks, k):
    ranks = np.asarray(ranks)
    return float(np.count_nonzero(ranks <= k) / ranks.size) if ranks.size else 0.0
