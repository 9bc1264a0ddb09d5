"""Pins for the oracle's generator, id mapping, sampling and table init."""
import os

import numpy as np
import pytest

from oracle import philox, sampling

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    with open(GOLD) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(x, 16) for x in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers_scalar():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, exp in rows:
        assert list(philox.philox4x32_10(ctr, key)) == exp


def test_philox_known_answers_numpy():
    for ctr, key, exp in _kat():
        out = philox.philox4x32_10_np(*[np.array([c], dtype=np.uint64) for c in ctr], key[0], key[1])
        assert [int(o[0]) for o in out] == exp


def test_philox_numpy_equals_scalar_on_random_counters():
    rng = np.random.default_rng(1)
    c = rng.integers(0, 1 << 32, size=(4, 200), dtype=np.uint64)
    k0, k1 = 0x12345678, 0x9ABCDEF0
    out = philox.philox4x32_10_np(c[0], c[1], c[2], c[3], k0, k1)
    for i in range(200):
        assert tuple(int(o[i]) for o in out) == philox.philox4x32_10([int(c[j, i]) for j in range(4)], (k0, k1))


def test_mulhi64_against_big_integers():
    rng = np.random.default_rng(2)
    x = rng.integers(0, 1 << 63, size=500, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, size=500, dtype=np.uint64)
    x[:3] = [0, (1 << 64) - 1, 1 << 63]
    for n in (1, 2, 3, 10_000, 14_951, 86_100_000, 1_460_000_000, (1 << 40) + 12345, (1 << 63) - 1):
        got = philox.mulhi64_np(x, n)
        for xi, gi in zip(x.tolist(), got.tolist()):
            assert gi == (xi * n) >> 64 == philox.mulhi64(xi, n)
            assert 0 <= gi < n


def test_random_words_follow_the_counter_layout():
    seed, step = 0xDEADBEEF12345678, (5 << 32) + 7
    x = sampling.random_words(seed, step, sampling.SIDE_DST, 3, 5)
    for c in range(3):
        for j in range(5):
            o = philox.philox4x32_10((j >> 1, 2 * c + 1, step & 0xFFFFFFFF, step >> 32),
                                     (seed & 0xFFFFFFFF, seed >> 32))
            w = (o[0] | (o[1] << 32)) if j % 2 == 0 else (o[2] | (o[3] << 32))
            assert int(x[c, j]) == w
    # the other side, another step and another seed all give different words
    assert not np.array_equal(x, sampling.random_words(seed, step, sampling.SIDE_SRC, 3, 5))
    assert not np.array_equal(x, sampling.random_words(seed, step + 1, sampling.SIDE_DST, 3, 5))
    assert not np.array_equal(x, sampling.random_words(seed + 1, step, sampling.SIDE_DST, 3, 5))


def test_uniform_negatives_chi_square():
    V = 50
    ns, nd = sampling.sample_negatives(0, 3, V, np.zeros(1, np.int32), np.zeros(1, np.int32), 40, 1000, 0)
    for ids in (ns, nd):
        assert ids.dtype == np.int32 and ids.shape == (40, 1000)
        assert ids.min() >= 0 and ids.max() < V
        cnt = np.bincount(ids.ravel(), minlength=V)
        chi2 = np.sum((cnt - 800.0) ** 2 / 800.0)
        assert chi2 < 100.0          # 49 dof: mean 49, 99.99th percentile ~ 95


def test_degree_negatives_follow_degree_and_come_first():
    rng = np.random.default_rng(3)
    V, E = 30, 5000
    w = np.arange(1, V + 1, dtype=np.float64) ** 2
    es = rng.choice(V, size=E, p=w / w.sum()).astype(np.int32)
    ed = rng.choice(V, size=E, p=w[::-1] / w.sum()).astype(np.int32)
    ns, nd = sampling.sample_negatives(7, 11, V, es, ed, 50, 400, 300)
    for ids, endpoints in ((ns, es), (nd, ed)):
        deg = np.bincount(endpoints, minlength=V).astype(np.float64)
        got = np.bincount(ids[:, :300].ravel(), minlength=V)
        exp = deg / deg.sum() * got.sum()
        mask = exp > 5
        chi2 = np.sum((got[mask] - exp[mask]) ** 2 / exp[mask])
        assert chi2 < 3.0 * mask.sum()
        assert got[deg == 0].sum() == 0
        # the uniform tail is far from degree-shaped
        tail = np.bincount(ids[:, 300:].ravel(), minlength=V)
        assert abs(tail - tail.mean()).max() < 6 * np.sqrt(tail.mean())
    # slot j of the degree part is endpoint[mulhi64(x, E)]
    x = sampling.random_words(7, 11, sampling.SIDE_SRC, 50, 400)
    assert ns[4, 17] == es[philox.mulhi64(int(x[4, 17]), E)]
    assert ns[4, 399] == philox.mulhi64(int(x[4, 399]), V)


def test_init_table_is_standard_normal_scaled():
    z = sampling.init_table(0, 0, 4000, 50, 0.001) / 0.001
    assert z.shape == (4000, 50)
    assert abs(z.mean()) < 4.0 / np.sqrt(z.size)
    assert abs(z.std() - 1.0) < 0.01
    assert abs(np.mean(z ** 4) - 3.0) < 0.1                # normal kurtosis
    assert abs(np.mean(z[:, 0::2].ravel()[:-1] * z[:, 0::2].ravel()[1:])) < 0.01
    # Box-Muller pair: radius and angle recover the two uniforms' ranges
    flat = z.reshape(-1)
    r2 = flat[0::2] ** 2 + flat[1::2] ** 2                # -2 ln u1, exponential(1/2)
    assert abs(np.mean(r2) - 2.0) < 0.02
    # another table / seed decorrelate
    z1 = sampling.init_table(0, 1, 4000, 50, 0.001) / 0.001
    assert abs(np.mean(z * z1)) < 0.01
    # prefix property: a smaller table is a prefix of the flattened stream
    small = sampling.init_table(0, 0, 10, 50, 0.001)
    assert np.array_equal(small.ravel(), (z * 0.001).ravel()[:500])
