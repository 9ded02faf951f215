"""Degrees, scaling and the normalized operator, written from the definitions.

Section II Step 2: D_ii = sum_j W_ij, L = D - W.  Section IV-B works with D^-1 W and assumes
D_ii > 0.  The symmetric form used throughout is S = D^-1/2 W D^-1/2 (similar to D^-1 W, same
eigenvalues) and L_sym = I - S; eigenvalue lambda of L_sym <-> theta = 1 - lambda of S.
"""
from __future__ import annotations

import numpy as np


def row_index(rowptr: np.ndarray) -> np.ndarray:
    """Row id of every stored entry."""
    n = rowptr.size - 1
    return np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))


def degrees(rowptr, col, val) -> np.ndarray:
    """d_i = sum_j W_ij  (Algorithm 2 steps 1-2: y = W 1)."""
    n = rowptr.size - 1
    return np.bincount(row_index(rowptr), weights=val, minlength=n).astype(np.float64)


def inv_sqrt_degrees(rowptr, col, val) -> np.ndarray:
    """s_i = d_i^-1/2; raises if some degree is not positive and finite (Section IV-B assumption)."""
    d = degrees(rowptr, col, val)
    if not np.all(np.isfinite(d)) or np.any(d <= 0.0):
        raise ValueError("every node must have a positive finite degree")
    return 1.0 / np.sqrt(d)


def apply_w(rowptr, col, val, x: np.ndarray) -> np.ndarray:
    """y = W x for a vector or an (n, b) array, entry by entry from the CSR triples."""
    n = rowptr.size - 1
    rows = row_index(rowptr)
    c = col.astype(np.int64)
    if x.ndim == 1:
        return np.bincount(rows, weights=val * x[c], minlength=n)
    out = np.empty((n, x.shape[1]))
    for t in range(x.shape[1]):
        out[:, t] = np.bincount(rows, weights=val * x[c, t], minlength=n)
    return out


def apply_s(rowptr, col, val, x: np.ndarray) -> np.ndarray:
    """y = S x = s * (W (s * x))."""
    s = inv_sqrt_degrees(rowptr, col, val)
    if x.ndim == 1:
        return s * apply_w(rowptr, col, val, s * x)
    return s[:, None] * apply_w(rowptr, col, val, s[:, None] * x)


class NormalizedOperator:
    """S as a callable, with the library CSR matvec as the primitive (same sums, faster)."""

    def __init__(self, rowptr, col, val):
        from scipy.sparse import csr_matrix
        n = rowptr.size - 1
        self.n = n
        self.s = inv_sqrt_degrees(rowptr, col, val)
        self.w = csr_matrix((np.asarray(val, dtype=np.float64), np.asarray(col), np.asarray(rowptr)),
                            shape=(n, n))
        self.count = 0

    def __call__(self, x: np.ndarray) -> np.ndarray:
        self.count += 1 if x.ndim == 1 else x.shape[1]
        if x.ndim == 1:
            return self.s * (self.w @ (self.s * x))
        return self.s[:, None] * (self.w @ (self.s[:, None] * x))


def dense_s(rowptr, col, val) -> np.ndarray:
    """Dense S (duplicates summed), for small n."""
    n = rowptr.size - 1
    s = inv_sqrt_degrees(rowptr, col, val)
    out = np.zeros((n, n))
    np.add.at(out, (row_index(rowptr), col.astype(np.int64)), val)
    return s[:, None] * out * s[None, :]


def dense_laplacian(rowptr, col, val) -> np.ndarray:
    """Dense L_sym = I - D^-1/2 W D^-1/2."""
    n = rowptr.size - 1
    return np.eye(n) - dense_s(rowptr, col, val)


def random_walk_vectors(rowptr, col, val, vec_sym: np.ndarray) -> np.ndarray:
    """Eigenvectors of the paper's L_n = D^-1 L (Section II Steps 2-3) from those of the symmetric form.

    If L_sym v = lambda v with L_sym = I - D^-1/2 W D^-1/2 then u = D^-1/2 v satisfies
    (I - D^-1 W) u = lambda u.  No renormalization: orthonormal v give D-orthonormal u (u_i^T D u_j = delta_ij)."""
    s = inv_sqrt_degrees(rowptr, col, val)
    return s[:, None] * vec_sym if vec_sym.ndim == 2 else s * vec_sym


def apply_random_walk_laplacian(rowptr, col, val, x: np.ndarray) -> np.ndarray:
    """y = L_n x = x - D^-1 (W x), entry by entry (Section II Step 2)."""
    d = degrees(rowptr, col, val)
    wx = apply_w(rowptr, col, val, x)
    return x - (wx / d[:, None] if x.ndim == 2 else wx / d)
