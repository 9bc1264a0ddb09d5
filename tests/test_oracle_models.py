"""Pins for the oracle's score functions and chunk blocks: closed forms,
identities, library routines and central finite differences."""
import numpy as np
import pytest

from oracle import models
from oracle.models import DISTMULT, COMPLEX, TRANSE, DOT, SIDE_SRC, SIDE_DST

ALL = (DISTMULT, COMPLEX, TRANSE, DOT)


def rows(rng, *shape):
    return rng.standard_normal(shape)


def test_distmult_closed_forms():
    rng = np.random.default_rng(0)
    s, r, d = rows(rng, 7, 6), rows(rng, 7, 6), rows(rng, 7, 6)
    f = models.score(DISTMULT, s, r, d)
    assert np.allclose(f, np.einsum("ek,ek,ek->e", s, r, d), rtol=1e-13)
    assert np.allclose(f, models.score(DISTMULT, d, r, s), rtol=1e-13)             # symmetric in s <-> d
    assert np.allclose(models.score(DISTMULT, s, np.ones_like(r), d), np.sum(s * d, axis=1))   # r = 1 -> Dot
    # the printed form theta_s^T diag(theta_r) theta_d
    assert np.isclose(f[3], s[3] @ np.diag(r[3]) @ d[3])


def test_dot_closed_forms():
    rng = np.random.default_rng(9)
    s, r, d = rows(rng, 7, 6), rows(rng, 7, 6), rows(rng, 7, 6)
    f = models.score(DOT, s, r, d)
    assert np.allclose(f, np.einsum("ek,ek->e", s, d), rtol=1e-13)
    assert np.allclose(f, models.score(DISTMULT, s, np.ones_like(r), d), rtol=1e-13)       # DistMult with r = 1
    assert np.array_equal(f, models.score(DOT, s, 5 * r, d))                               # no relation parameters
    assert np.all(models.score_grads(DOT, s, r, d)[1] == 0)


def test_complex_closed_forms():
    rng = np.random.default_rng(1)
    s, r, d = rows(rng, 5, 8), rows(rng, 5, 8), rows(rng, 5, 8)
    h = 4
    f = models.score(COMPLEX, s, r, d)
    sc, rc, dc = (x[:, :h] + 1j * x[:, h:] for x in (s, r, d))
    assert np.allclose(f, np.real(np.sum(sc * rc * np.conj(dc), axis=1)), rtol=1e-13)
    # four-term real expansion from the cited literature
    four = np.sum(s[:, :h] * r[:, :h] * d[:, :h] + s[:, h:] * r[:, :h] * d[:, h:]
                  + s[:, :h] * r[:, h:] * d[:, h:] - s[:, h:] * r[:, h:] * d[:, :h], axis=1)
    assert np.allclose(f, four, rtol=1e-12)
    # zero imaginary parts -> DistMult on the real half
    z = lambda x: np.concatenate([x[:, :h], np.zeros((5, h))], axis=1)
    assert np.allclose(models.score(COMPLEX, z(s), z(r), z(d)),
                       models.score(DISTMULT, s[:, :h], r[:, :h], d[:, :h]), rtol=1e-13)
    # real relation: symmetric; purely imaginary relation: antisymmetric
    rr = z(r)
    assert np.allclose(models.score(COMPLEX, s, rr, d), models.score(COMPLEX, d, rr, s))
    ri = np.concatenate([np.zeros((5, h)), r[:, h:]], axis=1)
    assert np.allclose(models.score(COMPLEX, s, ri, d), -models.score(COMPLEX, d, ri, s))


def test_transe_identities():
    rng = np.random.default_rng(2)
    s, r, d, t = rows(rng, 6, 5), rows(rng, 6, 5), rows(rng, 6, 5), rows(rng, 6, 5)
    f = models.score(TRANSE, s, r, d)
    assert np.all(f <= 0)
    assert np.allclose(models.score(TRANSE, s, r, s + r), 0.0, atol=1e-15)
    assert np.allclose(models.score(TRANSE, s + t, r, d + t), f, rtol=1e-12)
    assert np.allclose(models.score(TRANSE, -d, r, -s), f, rtol=1e-12)
    assert np.allclose(f, -np.linalg.norm(s + r - d, axis=1))
    # triangle inequality: |s+r-d| <= |s+r-x| + |x-d| = |s+r-x| + |x+0-d|
    x = rows(rng, 6, 5)
    assert np.all(-f <= -models.score(TRANSE, s, r, x) - models.score(TRANSE, x, 0 * r, d) + 1e-12)
    # scaling: f(c s, c r, c d) = |c| f
    assert np.allclose(models.score(TRANSE, 3 * s, 3 * r, 3 * d), 3 * f)


def _fd(fun, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h; fp = fun()
        x[i] = old - h; fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("model", ALL)
def test_score_grads_finite_differences(model):
    rng = np.random.default_rng(3 + model)
    s, r, d = rows(rng, 3, 6), rows(rng, 3, 6), rows(rng, 3, 6)
    gs, gr, gd = models.score_grads(model, s, r, d)
    w = rng.standard_normal(3)
    fun = lambda: float(np.sum(w * models.score(model, s, r, d)))
    assert np.allclose(_fd(fun, s), w[:, None] * gs, atol=1e-7)
    assert np.allclose(_fd(fun, r), w[:, None] * gr, atol=1e-7)
    assert np.allclose(_fd(fun, d), w[:, None] * gd, atol=1e-7)


def test_transe_gradient_is_zero_at_zero_distance():
    s = np.array([[1.0, 2.0]]); r = np.array([[0.5, -1.0]]); d = s + r
    for g in models.score_grads(TRANSE, s, r, d):
        assert np.all(g == 0) and np.all(np.isfinite(g))


@pytest.mark.parametrize("model", ALL)
@pytest.mark.parametrize("side", (SIDE_SRC, SIDE_DST))
def test_neg_block_is_the_score_function_entry_by_entry(model, side):
    rng = np.random.default_rng(10 * model + side)
    n, N, dim = 5, 7, 6
    S, R, D, Neg = rows(rng, n, dim), rows(rng, n, dim), rows(rng, n, dim), rows(rng, N, dim)
    A = models.neg_block(model, side, S, R, D, Neg)
    assert A.shape == (n, N)
    for e in range(n):
        for j in range(N):
            ref = models.score(model, S[e], R[e], Neg[j]) if side == SIDE_DST else models.score(model, Neg[j], R[e], D[e])
            assert np.isclose(A[e, j], ref, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("model", ALL)
@pytest.mark.parametrize("side", (SIDE_SRC, SIDE_DST))
def test_neg_block_backward_finite_differences(model, side):
    rng = np.random.default_rng(100 + 10 * model + side)
    n, N, dim = 3, 4, 6
    S, R, D, Neg = rows(rng, n, dim), rows(rng, n, dim), rows(rng, n, dim), rows(rng, N, dim)
    P = rng.standard_normal((n, N))
    gS, gR, gD, gNeg = models.neg_block_backward(model, side, S, R, D, Neg, P)
    fun = lambda: float(np.sum(P * models.neg_block(model, side, S, R, D, Neg)))
    assert np.allclose(_fd(fun, S), gS, atol=2e-7)
    assert np.allclose(_fd(fun, R), gR, atol=2e-7)
    assert np.allclose(_fd(fun, D), gD, atol=2e-7)
    assert np.allclose(_fd(fun, Neg), gNeg, atol=2e-7)
    # the uncorrupted endpoint's own row does not enter the block
    assert np.all((gD if side == SIDE_DST else gS) == 0)


def test_transe_block_handles_a_negative_equal_to_the_target():
    S = np.array([[1.0, 0.0]]); R = np.array([[0.0, 1.0]]); D = np.array([[3.0, 3.0]])
    Neg = np.array([[1.0, 1.0], [0.0, 0.0]])              # first negative == s + r exactly
    A = models.neg_block(TRANSE, SIDE_DST, S, R, D, Neg)
    assert A[0, 0] == 0.0 and np.isclose(A[0, 1], -np.sqrt(2.0))
    out = models.neg_block_backward(TRANSE, SIDE_DST, S, R, D, Neg, np.ones((1, 2)))
    assert all(np.all(np.isfinite(g)) for g in out)
    assert np.allclose(out[3][0], 0.0)
