"""Dense block steps of the Lanczos process, by their definitions (numpy fp64).  Test infrastructure.

* ``cgs2_block``: classical Gram-Schmidt applied twice to a block W against an orthonormal Q
  (the reorthogonalization inside each Lanczos step, Section IV-B).
* ``rotate``: Ritz vectors / restart rotation V Y (FindEigenvectors of Algorithm 3).
"""
from __future__ import annotations

import numpy as np


def cgs2_block(q: np.ndarray, w: np.ndarray):
    """Returns (W orthogonalised against the columns of q, H1 + H2)."""
    w = w.copy()
    h1 = q.T @ w
    w -= q @ h1
    h2 = q.T @ w
    w -= q @ h2
    return w, h1 + h2


def rotate(v: np.ndarray, y: np.ndarray) -> np.ndarray:
    return v @ y


def chebyshev_filter(rowptr, col, val, x: np.ndarray, a: float, degree: int) -> np.ndarray:
    """T_d(g(S)) x with g(S) = (2 S - (a - 1) I) / (a + 1), the affine image of [-1, a] in [-1, 1].

    The start vector of Algorithm 3 is free; the GPU solver filters its re-injection blocks with this polynomial.
    Written as the three-term recurrence of the Chebyshev polynomials of the first kind,
    T_0 = 1, T_1(t) = t, T_{i+1}(t) = 2 t T_i(t) - T_{i-1}(t), with S applied entry by entry."""
    from . import laplacian

    def g(v):
        return (2.0 * laplacian.apply_s(rowptr, col, val, v) - (a - 1.0) * v) / (a + 1.0)

    y_prev = np.array(x, dtype=np.float64, copy=True)
    if degree == 0:
        return y_prev
    y_cur = g(y_prev)
    for _ in range(degree - 1):
        y_prev, y_cur = y_cur, 2.0 * g(y_cur) - y_prev
    return y_cur
