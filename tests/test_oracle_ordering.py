"""Pins for the oracle's BETA ordering and buffer simulator: the values the paper states, Eq. 2 / Eq. 3,
and structural invariants."""
import itertools
import os

import pytest

from oracle import ordering

CASES = [(4, 2), (6, 3), (8, 2), (8, 4), (16, 4), (32, 8), (10, 3), (9, 5), (12, 5), (7, 7), (5, 4), (64, 16)]


def test_values_stated_in_the_paper():
    gold = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "beta_examples.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                gold[(int(line[0]), int(line[1]), line[2])] = line[3]
    # p = 4, c = 2: five misses
    seq = ordering.beta_buffer_sequence(4, 2)
    assert len(seq) - 1 == int(gold[(4, 2, "beta_misses")]) == ordering.beta_swap_count(4, 2)
    assert ordering.simulate_buffer(ordering.edge_bucket_order(seq, 4), 2) - 2 == 5
    # p = 6, c = 3: the sets of fixed leading partitions, in order
    seq = ordering.beta_buffer_sequence(6, 3)
    fixed = []
    for buf in seq:
        lead = sorted(buf[:2])
        if not fixed or fixed[-1] != lead:
            fixed.append(lead)
    stable = [s for s in fixed if s in ([0, 1], [2, 3])]
    assert stable == [[0, 1], [2, 3]]
    assert seq[-1][0] == 5 and set(seq[-1]) == {5, 3, 4}      # {2,3} finally replaced (as far as disk allows) by {5}
    assert len(seq) - 1 == 7 == ordering.beta_swap_count(6, 3) and ordering.swap_lower_bound(6, 3) == 6


@pytest.mark.parametrize("p,c", CASES)
def test_buffer_sequence_invariants(p, c):
    seq = ordering.beta_buffer_sequence(p, c)
    assert seq[0] == list(range(c))
    for a, b in zip(seq, seq[1:]):
        assert len(set(b)) == c
        assert len(set(a) ^ set(b)) == 2                      # successive buffers differ by one swapped partition
    together = set()
    for buf in seq:
        together.update(itertools.combinations(sorted(buf), 2))
    assert len(together) == p * (p - 1) // 2                  # every pair meets in the buffer at least once
    assert len(seq) - 1 == ordering.beta_swap_count(p, c)     # Eq. 3
    assert ordering.swap_lower_bound(p, c) <= len(seq) - 1    # Eq. 2


@pytest.mark.parametrize("p,c", CASES)
@pytest.mark.parametrize("seed", (None, 7))
def test_edge_bucket_order_and_simulated_swaps(p, c, seed):
    seq = ordering.beta_buffer_sequence(p, c)
    order = ordering.edge_bucket_order(seq, p, seed)
    assert sorted(order) == [(i, j) for i in range(p) for j in range(p)]      # every bucket exactly once
    # buckets become available buffer by buffer: replaying the order through the sequence never misses
    pos = 0
    for buf in seq:
        while pos < len(order) and order[pos][0] in buf and order[pos][1] in buf:
            pos += 1
    assert pos == len(order)
    loads = ordering.simulate_buffer(order, c)
    assert loads - c == ordering.beta_swap_count(p, c)
    assert loads - c >= ordering.swap_lower_bound(p, c)


def test_shuffle_is_a_seeded_permutation_within_buffers():
    seq = ordering.beta_buffer_sequence(8, 4)
    a = ordering.edge_bucket_order(seq, 8, 1)
    b = ordering.edge_bucket_order(seq, 8, 1)
    c = ordering.edge_bucket_order(seq, 8, 2)
    plain = ordering.edge_bucket_order(seq, 8)
    assert a == b and a != c and a != plain
    assert sorted(a[:16]) == sorted(plain[:16])               # the first buffer's 16 buckets stay in front
    # a naive row-major order needs far more swaps than BETA
    rowmajor = [(i, j) for i in range(8) for j in range(8)]
    assert ordering.simulate_buffer(rowmajor, 4) - 4 > ordering.beta_swap_count(8, 4)


def test_closed_forms_small_table():
    # Eq. 2 by hand: p=4,c=2: (6-1)/1 = 5; p=6,c=3: ceil(12/2) = 6; p=8,c=4: ceil(22/3) = 8
    assert [ordering.swap_lower_bound(*pc) for pc in ((4, 2), (6, 3), (8, 4))] == [5, 6, 8]
    # Eq. 3 by hand: p=8,c=4: x=1 -> 4 + 2*(4 - 1.5) = 9 ; p=c: 0
    assert ordering.beta_swap_count(8, 4) == 9 and ordering.beta_swap_count(7, 7) == 0
