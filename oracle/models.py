"""Score functions f(theta_s, theta_r, theta_d) and their partial derivatives
(oracle side; test infrastructure).  All arithmetic in fp64.

* DistMult: f = theta_s^T diag(theta_r) theta_d, the one formula Sec. 2.1 prints.
* ComplEx: only cited in Sec. 2.1 / used in Sec. 5.1.  Taken from the cited
  literature: f = Re(sum_k s_k r_k conj(d_k)) over dim/2 complex numbers; a row of
  ``dim`` floats stores the real parts first, then the imaginary parts.
* TransE: only cited in Sec. 2.1 ("linear score functions").  Reading taken:
  f = -||s + r - d||_2 (not squared); the derivative at distance 0 is taken as 0.
* Dot: f = theta_s . theta_d, "a dot product between the node embeddings of an edge" (Sec. 5.1,
  "Embedding Models"); it has no relation parameters.

``neg_block`` / ``neg_block_backward`` evaluate one chunk's positives against the
chunk's shared negative set: a[e, j] = f(s_e, r_e, n_j) when the negatives replace
the destination, b[e, j] = f(m_j, r_e, d_e) when they replace the source.  A
matrix product is used as a step where the score is bilinear in the negative;
no tiling or fusion beyond that.
"""
import numpy as np

DISTMULT = 0
COMPLEX = 1
TRANSE = 2
DOT = 3

SIDE_SRC = 0   # negatives replace the source
SIDE_DST = 1   # negatives replace the destination


def _cplx(x):
    h = x.shape[-1] // 2
    return x[..., :h] + 1j * x[..., h:]


def _real(z):
    return np.concatenate([z.real, z.imag], axis=-1)


def score(model, s, r, d):
    """f for broadcastable row arrays (..., dim) -> (...)."""
    s = np.asarray(s, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    d = np.asarray(d, dtype=np.float64)
    if model == DISTMULT:
        return np.sum(s * r * d, axis=-1)
    if model == COMPLEX:
        return np.sum(_cplx(s) * _cplx(r) * np.conj(_cplx(d)), axis=-1).real
    if model == TRANSE:
        return -np.sqrt(np.sum((s + r - d) ** 2, axis=-1))
    if model == DOT:
        return np.sum(s * d + 0.0 * r, axis=-1)
    raise ValueError("unknown model %r" % (model,))


def score_grads(model, s, r, d):
    """(df/ds, df/dr, df/dd), each shaped like the broadcast rows."""
    s = np.asarray(s, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    d = np.asarray(d, dtype=np.float64)
    if model == DISTMULT:
        return r * d, s * d, s * r
    if model == COMPLEX:
        sc, rc, dc = _cplx(s), _cplx(r), _cplx(d)
        # For a real function Re(z c) of z = x + iy, (d/dx, d/dy) packs as conj(c).
        return (_real(np.conj(rc) * dc),          # f = Re(s * (r conj d))
                _real(np.conj(sc) * dc),          # f = Re(r * (s conj d))
                _real(sc * rc))                   # f = Re(conj(d) * (s r)) -> s r
    if model == TRANSE:
        diff = s + r - d
        dist = np.sqrt(np.sum(diff ** 2, axis=-1, keepdims=True))
        unit = np.divide(diff, dist, out=np.zeros_like(diff), where=dist > 0)
        return -unit, -unit, unit
    if model == DOT:
        return d + 0.0 * r, 0.0 * (s + r + d), s + 0.0 * r
    raise ValueError("unknown model %r" % (model,))


def neg_block(model, side, S, R, D, Neg):
    """Scores of every edge of a chunk (rows S, R, D: (n, dim)) against the chunk's
    negatives Neg (N, dim): returns (n, N)."""
    if model == DISTMULT:
        q = S * R if side == SIDE_DST else R * D
        return q @ Neg.T
    if model == DOT:
        return (S if side == SIDE_DST else D) @ Neg.T
    if model == COMPLEX:
        if side == SIDE_DST:
            return ((_cplx(S) * _cplx(R)) @ np.conj(_cplx(Neg)).T).real
        return (_cplx(Neg) @ (_cplx(R) * np.conj(_cplx(D))).T).real.T
    if model == TRANSE:
        out = np.empty((S.shape[0], Neg.shape[0]), dtype=np.float64)
        for e in range(S.shape[0]):
            if side == SIDE_DST:
                diff = (S[e] + R[e])[None, :] - Neg
            else:
                diff = Neg + (R[e] - D[e])[None, :]
            out[e] = -np.sqrt(np.sum(diff ** 2, axis=1))
        return out
    raise ValueError("unknown model %r" % (model,))


def neg_block_backward(model, side, S, R, D, Neg, P):
    """Given P[e, j] = dL/d(score[e, j]) returns (gS, gR, gD, gNeg): the sums
    sum_j P[e,j] df/d(row of e) and sum_e P[e,j] df/d(n_j)."""
    n, dim = S.shape
    zero = np.zeros((n, dim), dtype=np.float64)
    if model == DISTMULT:
        if side == SIDE_DST:
            gq = P @ Neg                      # d/d(s*r)
            return gq * R, gq * S, zero, P.T @ (S * R)
        gq = P @ Neg                          # d/d(r*d)
        return zero, gq * D, gq * R, P.T @ (R * D)
    if model == DOT:
        if side == SIDE_DST:
            return P @ Neg, zero, zero, P.T @ S
        return zero, zero, P @ Neg, P.T @ D
    if model == COMPLEX:
        sc, rc, dc, nc = _cplx(S), _cplx(R), _cplx(D), _cplx(Neg)
        if side == SIDE_DST:
            # a = Re(u conj(n)), u = s r: packed gradient w.r.t. u is n, w.r.t. n is u.
            gu = P @ nc
            return _real(np.conj(rc) * gu), _real(np.conj(sc) * gu), zero, _real(P.T @ (sc * rc))
        # b = Re(m conj(w)), w = conj(r) d: packed gradient w.r.t. w is m, w.r.t. m is w.
        gw = P @ nc
        return zero, _real(np.conj(gw) * dc), _real(rc * gw), _real(P.T @ (np.conj(rc) * dc))
    if model == TRANSE:
        gS = np.zeros((n, dim)); gR = np.zeros((n, dim)); gD = np.zeros((n, dim))
        gNeg = np.zeros_like(Neg)
        for e in range(n):
            if side == SIDE_DST:
                diff = (S[e] + R[e])[None, :] - Neg      # f = -|diff|
            else:
                diff = Neg + (R[e] - D[e])[None, :]
            dist = np.sqrt(np.sum(diff ** 2, axis=1, keepdims=True))
            unit = np.divide(diff, dist, out=np.zeros_like(diff), where=dist > 0)
            w = P[e][:, None] * unit                     # P * d|diff|/d(diff)
            tot = w.sum(axis=0)
            if side == SIDE_DST:
                gS[e] -= tot; gR[e] -= tot; gNeg += w
            else:
                gR[e] -= tot; gD[e] += tot; gNeg -= w
        return gS, gR, gD, gNeg
    raise ValueError("unknown model %r" % (model,))
