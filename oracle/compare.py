"""Measures used by the parity tests.  They recompute everything from the CSR triples and the
vectors under test in fp64; nothing is taken from a solver's own estimates."""
from __future__ import annotations

import numpy as np

from .laplacian import NormalizedOperator


def residual_norms(rowptr, col, val, lam: np.ndarray, vec: np.ndarray) -> np.ndarray:
    """||L v_i - lambda_i v_i||_2 per pair, L = I - S."""
    op = NormalizedOperator(rowptr, col, val)
    lv = vec - op(vec)
    return np.linalg.norm(lv - vec * lam[None, :], axis=0)


def orthonormality_defect(vec: np.ndarray) -> float:
    g = vec.T @ vec
    return float(np.max(np.abs(g - np.eye(g.shape[0]))))


def principal_angles(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Principal angles (radians, ascending) between span(a) and span(b); accurate for small
    angles (sine-based)."""
    qa, _ = np.linalg.qr(a)
    qb, _ = np.linalg.qr(b)
    if qa.shape[1] > qb.shape[1]:
        qa, qb = qb, qa
    # sines from the part of qa outside span(qb) (dimension of the smaller space)
    resid = qa - qb @ (qb.T @ qa)
    sines = np.linalg.svd(resid, compute_uv=False)
    return np.arcsin(np.clip(np.sort(sines), 0.0, 1.0))


def containment_defect(x: np.ndarray, basis: np.ndarray) -> np.ndarray:
    """|| (I - N N^T) x_i ||_2 per column, N an orthonormal basis of span(basis)."""
    qn, _ = np.linalg.qr(basis)
    r = x - qn @ (qn.T @ x)
    return np.linalg.norm(r, axis=0)


def separated_clusters(lam_ext: np.ndarray, k: int, r_sum: float, ratio: float = 5e-6):
    """Split indices 0..k-1 of the ascending eigenvalues ``lam_ext`` (length > k: the oracle also
    supplies lambda_{k+1}) into maximal runs whose gaps to both neighbours satisfy
    r_sum / gap <= ratio (Davis-Kahan: the subspace of such a run is determined to that angle).
    Returns a list of (start, stop) half-open index ranges that are separated, skipping a last run
    that is not separated from lambda_{k+1}."""
    gaps = np.diff(lam_ext[: k + 1])
    cut = [i + 1 for i in range(k) if gaps[i] > 0 and r_sum / gaps[i] <= ratio]
    runs, start = [], 0
    for c in cut:
        if c > start:
            runs.append((start, c))
        start = c
    return [(a, b) for a, b in runs if b <= k]
