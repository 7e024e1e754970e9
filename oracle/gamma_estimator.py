"""Setting the relaxation parameter gamma from a confidence level p (Section 3.2) -- oracle
side, test infrastructure only (see oracle/__init__.py).  Plain numpy in float64.

By the lemma of Section 3.2 the confidence level of Equation 3 is p = P(gamma <= 1 - cos(theta)),
theta being the angle at the landmark l between x - l and q - l.  For a data vector x the value
gamma_x(p) is therefore read off the distribution of 1 - Z, Z = cos(x - l, q - l): the largest
gamma that at least a fraction p of the queries satisfy; one global gamma = the smallest
gamma_x over a sample of data vectors (end of Section 3.2).

Two ways to get the distribution, as in the paper:
  * empirical: 1 - Z computed for sampled data vectors against sampled queries;
  * standard-normal queries: Z^2 = A / (A + B + C) with A = (Q1 + h1)^2, B = (Q2 - h2)^2,
    C = sum of the squares of the remaining coordinates, h1 = (x - l).l / |x - l|,
    h2 = sqrt(|l|^2 - h1^2) (the theorem giving Z^2), and the CDF of 1 - Z obtained from the
    CDF of Z^2 by the transform theorem.  The normal variates are inputs, never drawn here.

Readings (the text leaves them open or contradicts itself):
  * with Q sampled values v[0] <= ... <= v[Q-1] of 1 - Z, gamma_x(p) = v[Q - m],
    m = min(Q, max(1, ceil(p * Q))): the m-th largest value, so that exactly m of the Q sampled
    queries satisfy gamma <= 1 - cos(theta); p = 1 gives the smallest value;
  * the sum C runs over coordinates 3..d, i.e. d - 2 terms (the text names chi_{d-3} next to a
    sum of d - 2 squares; the sum is what the proof derives);
  * the transform theorem halves P(Z^2 >= (1-y)^2) between the two signs of Z, i.e. it
    treats Z as symmetric about 0; it is applied as printed (exact for a landmark at the
    origin, an approximation otherwise: the test measures it only where it is exact);
  * a data vector equal to its landmark (x - l = 0), or a query equal to the landmark, has no
    angle: 1 - Z is taken as 1 (cos = 0).
"""
from __future__ import annotations

import math

import numpy as np


def landmarks(codes: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """PQ reconstructions (Section 3.1: the landmark of x), float64 [n][d]."""
    M = codebooks.shape[0]
    return np.concatenate([codebooks[j][codes[:, j]] for j in range(M)], axis=1).astype(np.float64)


def one_minus_cos(x: np.ndarray, l: np.ndarray, queries: np.ndarray) -> np.ndarray:
    """1 - cos(x - l, q - l) for one data vector against every query."""
    u = x.astype(np.float64) - l.astype(np.float64)
    w = queries.astype(np.float64) - l.astype(np.float64)[None, :]
    nu = math.sqrt(float(u @ u))
    nw = np.sqrt((w * w).sum(axis=1))
    den = nu * nw
    z = np.divide(w @ u, den, out=np.zeros_like(den), where=den > 0)
    return 1.0 - z


def rank_for_p(p: float, count: int) -> int:
    """Index into the ascending sample of the value returned for confidence p."""
    m = min(count, max(1, math.ceil(float(np.float32(p)) * count)))
    return count - m


def gamma_from_sample(values: np.ndarray, p: float) -> float:
    v = np.sort(np.asarray(values, dtype=np.float64))
    return float(v[rank_for_p(p, v.shape[0])])


def estimate_gamma_empirical(base, codes, codebooks, rows, queries, p):
    """(gamma, gamma_x[len(rows)]) from sampled data vectors (positions `rows`) and queries."""
    lm = landmarks(codes[rows], codebooks)
    gx = np.array([gamma_from_sample(one_minus_cos(base[r], lm[i], queries), p)
                   for i, r in enumerate(rows)], dtype=np.float64)
    return float(gx.min()), gx


def h1_h2(x: np.ndarray, l: np.ndarray):
    u = x.astype(np.float64) - l.astype(np.float64)
    l64 = l.astype(np.float64)
    h1 = float(u @ l64) / math.sqrt(float(u @ u))
    h2 = math.sqrt(max(float(l64 @ l64) - h1 * h1, 0.0))
    return h1, h2


def z2_samples(h1: float, h2: float, normals: np.ndarray) -> np.ndarray:
    """Z^2 = A / (A + B + C) for rows of standard-normal variates [count][d] (only the
    distribution of the row matters: coordinate 0 plays Q1, coordinate 1 plays Q2)."""
    a = (normals[:, 0] + h1) ** 2
    b = (normals[:, 1] - h2) ** 2
    c = (normals[:, 2:] ** 2).sum(axis=1)
    return a / (a + b + c)


def cdf_one_minus_z_from_z2(z2_sorted: np.ndarray, y: np.ndarray) -> np.ndarray:
    """The transform theorem: F_{1-Z}(y) = 1/2 -+ F_{Z^2}((1-y)^2)/2 for y <= 1 / y > 1,
    with F_{Z^2} the empirical CDF of the given sorted sample."""
    f = np.searchsorted(z2_sorted, (1.0 - y) ** 2, side="right") / z2_sorted.shape[0]
    return np.where(y <= 1.0, 0.5 - 0.5 * f, 0.5 + 0.5 * f)


def gamma_normal_queries(x: np.ndarray, l: np.ndarray, normals: np.ndarray, p: float,
                         grid: int = 20001) -> float:
    """gamma_x(p) for standard-normal queries: the largest y on a grid over [0, 2] whose
    CDF value F_{1-Z}(y) is at most 1 - p (so that P(1 - Z >= y) >= p up to the grid step)."""
    h1, h2 = h1_h2(x, l)
    z2 = np.sort(z2_samples(h1, h2, normals.astype(np.float64)))
    y = np.linspace(0.0, 2.0, grid)
    f = cdf_one_minus_z_from_z2(z2, y)
    ok = np.flatnonzero(f <= 1.0 - float(np.float32(p)) + 1e-12)
    return float(y[ok[-1]]) if ok.size else 0.0
