"""Plain definition: the k smallest eigenpairs of the dense normalized Laplacian (Section II
Step 3 with the zero eigenvalues included, Section IV-B first paragraph)."""
from __future__ import annotations

import numpy as np

from .laplacian import dense_laplacian


def full_spectrum(rowptr, col, val):
    """All eigenvalues (ascending) and orthonormal eigenvectors of L_sym."""
    lap = dense_laplacian(rowptr, col, val)
    lap = 0.5 * (lap + lap.T)
    return np.linalg.eigh(lap)


def smallest_eigenpairs(rowptr, col, val, k: int):
    """(lambda[0:k], V[:, 0:k]) counted with multiplicity."""
    lam, vec = full_spectrum(rowptr, col, val)
    return lam[:k].copy(), vec[:, :k].copy()
