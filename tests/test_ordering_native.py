"""The library's host-side BETA ordering and buffer simulator against the oracle (bit exact; no GPU)."""
import os

import numpy as np
import pytest

import paper_2101_08358_amd as mar
from oracle import ordering

CASES = [(4, 2), (6, 3), (8, 2), (8, 4), (16, 4), (32, 8), (10, 3), (9, 5), (12, 5), (7, 7), (5, 4), (64, 16)]


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(mar.library_path()):
        from paper_2101_08358_amd import build
        build.build()
    mar.load_library()


@pytest.mark.parametrize("p,c", CASES)
def test_buffer_sequence_and_closed_forms(p, c):
    seq = mar.mar_beta_buffer_sequence(p, c)
    assert seq.tolist() == ordering.beta_buffer_sequence(p, c)
    assert mar.mar_beta_swap_count(p, c) == ordering.beta_swap_count(p, c) == seq.shape[0] - 1
    assert mar.mar_swap_lower_bound(p, c) == ordering.swap_lower_bound(p, c)


@pytest.mark.parametrize("p,c", CASES)
@pytest.mark.parametrize("seed", (None, 0, 0xABCDEF0123456789))
def test_edge_bucket_order_and_simulation(p, c, seed):
    got = mar.mar_beta_edge_bucket_order(p, c, seed is not None, seed or 0)
    exp = ordering.edge_bucket_order(ordering.beta_buffer_sequence(p, c), p, seed)
    assert [tuple(x) for x in got.tolist()] == exp
    loads = mar.mar_buffer_simulate(p, c, got)
    assert loads == ordering.simulate_buffer(exp, c)
    assert loads - c == mar.mar_beta_swap_count(p, c)


def test_simulator_on_other_orders_matches_oracle():
    rng = np.random.default_rng(0)
    for p, c in ((8, 3), (12, 4), (20, 5)):
        order = [(i, j) for i in range(p) for j in range(p)]
        for _ in range(3):
            perm = rng.permutation(len(order))
            o = [order[k] for k in perm]
            assert mar.mar_buffer_simulate(p, c, np.array(o, dtype=np.int32)) == ordering.simulate_buffer(o, c)
        assert mar.mar_buffer_simulate(p, c, np.array(order, dtype=np.int32)) == ordering.simulate_buffer(order, c)


def test_argument_errors():
    assert mar.mar_swap_lower_bound(3, 1) == -1 and mar.mar_beta_swap_count(2, 3) == -1
    with pytest.raises(mar.MarError):
        mar.mar_beta_buffer_sequence(3, 5)
    with pytest.raises(mar.MarError):
        mar.mar_buffer_simulate(4, 2, np.array([[0, 9]], dtype=np.int32))
