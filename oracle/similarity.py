"""Similarity-graph construction (Section IV-A: the three similarity measures and Algorithm 1; Algorithm 2 step 4, the
COO to CSR conversion).  Plain numpy fp64 definitions, one edge at a time in vector form.

The exponential-decay measure is printed in the paper without the minus sign and the square; the reading taken is
exp(-|x_i - x_j|^2 / (2 sigma^2)) (a similarity that decays with distance).

Test infrastructure only."""
from __future__ import annotations

import numpy as np

CROSS_CORRELATION, COSINE, EXP_DECAY = 0, 1, 2


def row_means(x: np.ndarray) -> np.ndarray:
    """Algorithm 1 step 4: X_average(i) = (1/d) sum_j X_ij."""
    return x.sum(axis=1) / x.shape[1]


def centered_norms(x: np.ndarray) -> np.ndarray:
    """Algorithm 1 step 5: 2-norm of every row after its mean was subtracted."""
    xc = x - row_means(x)[:, None]
    return np.sqrt((xc * xc).sum(axis=1))


def edge_similarity(x: np.ndarray, u: np.ndarray, v: np.ndarray, measure: int, sigma: float = 1.0) -> np.ndarray:
    """Algorithm 1 step 6 for the listed pairs (u_e, v_e)."""
    xu, xv = x[u], x[v]
    if measure == CROSS_CORRELATION:
        m = row_means(x)
        nrm = centered_norms(x)
        cu, cv = xu - m[u][:, None], xv - m[v][:, None]
        return (cu * cv).sum(axis=1) / (nrm[u] * nrm[v])
    if measure == COSINE:
        nrm = np.sqrt((x * x).sum(axis=1))
        return (xu * xv).sum(axis=1) / (nrm[u] * nrm[v])
    if measure == EXP_DECAY:
        diff = xu - xv
        return np.exp(-(diff * diff).sum(axis=1) / (2.0 * sigma * sigma))
    raise ValueError(measure)


def coo_to_dense(row, col, val, n: int, symmetrize: bool) -> np.ndarray:
    """The matrix a COO list stands for, entry by entry (duplicates add up); with `symmetrize` every listed pair
    (r, c), r != c, also stands for (c, r)."""
    a = np.zeros((n, n))
    for r, c, w in zip(row, col, val):
        a[r, c] += w
        if symmetrize and r != c:
            a[c, r] += w
    return a


def csr_rows_sorted(rowptr, col) -> bool:
    return all(np.all(np.diff(col[rowptr[i]:rowptr[i + 1]]) >= 0) for i in range(rowptr.size - 1))
