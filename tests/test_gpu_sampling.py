"""GPU parity (bit exact): negative ids and table initialisation against the oracle."""
import numpy as np
import pytest
import torch

import paper_2101_08358_amd as mar
from oracle import sampling

pytestmark = pytest.mark.gpu


def _sample_both(V, E, C, N, Ndeg, seed, step, rng):
    es = rng.integers(0, V, E).astype(np.int32)
    ed = rng.integers(0, V, E).astype(np.int32)
    # the sampler only needs num_nodes, but a context owns real tables: keep them narrow when V is large
    tr = mar.Trainer(V, 1, 1 if V > 100000 else 8, 0, C, C, N, Ndeg, seed=seed)
    d_es, d_ed = torch.from_numpy(es).to(tr.device), torch.from_numpy(ed).to(tr.device)
    tr.sample_negatives(step, d_es, d_ed)
    torch.cuda.synchronize()
    got = tr.neg_src.cpu().numpy().reshape(C, N), tr.neg_dst.cpu().numpy().reshape(C, N)
    tr.close()
    exp = sampling.sample_negatives(seed, step, V, es, ed, C, N, Ndeg)
    return got, exp


@pytest.mark.parametrize("V,E,C,N,Ndeg,seed,step", (
    (10_000, 100_000, 10, 100, 0, 0, 0),
    (14_951, 483_142, 10, 1000, 100, 0, 48),
    (41_600_000, 3_000_000, 50, 1000, 500, 0xDEADBEEFCAFEF00D, (1 << 40) + 12345),
    (7, 5, 3, 33, 33, 5, 1),                         # odd N, all degree-based
    (2_000_000_000, 1000, 2, 17, 3, 9, (1 << 62) + 1),   # id range close to 2^31
))
def test_negative_ids_bit_exact(V, E, C, N, Ndeg, seed, step):
    print("case", V, E, C, N, Ndeg, flush=True)
    rng = np.random.default_rng(1)
    got, exp = _sample_both(V, E, C, N, Ndeg, seed, step, rng)
    assert np.array_equal(got[0], exp[0])
    assert np.array_equal(got[1], exp[1])


def test_sampling_is_stateless_and_step_dependent():
    tr = mar.Trainer(1000, 1, 8, 0, 10, 10, 50, 0, seed=4)
    tr.sample_negatives(3)
    a = tr.neg_src.clone(), tr.neg_dst.clone()
    tr.sample_negatives(4)
    b = tr.neg_src.clone(), tr.neg_dst.clone()
    tr.sample_negatives(3)
    torch.cuda.synchronize()
    assert torch.equal(a[0], tr.neg_src) and torch.equal(a[1], tr.neg_dst)
    assert not torch.equal(a[0], b[0]) and not torch.equal(a[0], a[1])
    tr.close()


@pytest.mark.parametrize("V,R,dim,seed", ((1000, 7, 50, 0), (333, 3, 17, 12345678901234567), (20000, 40, 400, 3)))
def test_table_init_matches_oracle(V, R, dim, seed):
    tr = mar.Trainer(V, R, dim, 0, 8, 2, 4, 0, init_std=0.001, seed=seed)
    torch.cuda.synchronize()
    for table, got in ((0, tr.node_emb), (1, tr.rel_emb)):
        exp = sampling.init_table(seed, table, got.shape[0], dim, np.float32(0.001))
        err = np.max(np.abs(got.cpu().numpy().astype(np.float64) - exp))
        assert err <= 1e-5 * 0.001, err          # fp32 log / sqrt / sincos against fp64: absolute, in units of std
    assert torch.count_nonzero(tr.node_state).item() == 0 and torch.count_nonzero(tr.rel_state).item() == 0
    tr.close()
