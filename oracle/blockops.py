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
