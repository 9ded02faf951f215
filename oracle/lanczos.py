"""Single-vector Lanczos with full reorthogonalization, thick restart, locking and random
re-injection: the iterative route to the plain definition in ``dense.py``.

What the paper fixes (Section IV-B, Algorithm 3): the wanted pairs are the largest eigenvalues
of the degree-normalized similarity matrix (equivalently the smallest of the normalized
Laplacian), found by a restarted Lanczos process whose only contact with the matrix is one
sparse matrix-vector product per step, whose per-step dense work is the reorthogonalization
against the m stored Lanczos vectors, whose per-restart work is the eigendecomposition of the
m x m projected matrix, and whose last act is forming the Ritz vectors (FindEigenvectors).

What the paper leaves open, and the reading taken here:

* operator: the symmetric S = D^-1/2 W D^-1/2 (Lanczos needs a symmetric operator; same
  eigenvalues as D^-1 W); wanted = algebraically largest theta of S, lambda = 1 - theta;
* reorthogonalization: classical Gram-Schmidt against all locked and Lanczos vectors, twice;
* convergence of a Ritz pair: residual estimate |beta_j * (last component of its T-eigenvector)|
  <= tol (the norm of S is 1, so absolute = relative);
* multiple eigenvalues: a Krylov space of one start vector holds one copy of a multiple
  eigenvalue, so the process runs in phases.  Each phase starts from a fresh seeded random
  vector made orthogonal to everything locked so far, runs until its leading Ritz pair(s)
  converge, and locks them.  It stops when at least k pairs are locked and a whole new phase
  finds nothing larger than the k-th largest locked theta (+ tol);
* restart: thick restart (keep the leading Ritz vectors and the residual vector; the projected
  matrix becomes diagonal plus one coupling row);
* maxiter: number of restart cycles (phase starts + thick restarts);
* the result is refined by a Rayleigh-Ritz step over the span of all locked vectors.
"""
from __future__ import annotations

import numpy as np

from .laplacian import NormalizedOperator


def _cgs2(w: np.ndarray, bases) -> list:
    """Classical Gram-Schmidt, applied twice, of w against the columns of each array in ``bases``.
    Returns the summed coefficients per basis; w is updated in place."""
    coeffs = [np.zeros(b.shape[1]) for b in bases]
    for _ in range(2):
        hs = [b.T @ w for b in bases]          # all coefficients from the same w (classical GS)
        for b, h in zip(bases, hs):
            w -= b @ h
        for c, h in zip(coeffs, hs):
            c += h
    return coeffs


def lanczos_smallest(rowptr, col, val, k: int, tol: float, m: int | None = None, seed: int = 0,
                     maxiter: int = 100000, return_info: bool = False):
    """k smallest eigenpairs of I - D^-1/2 W D^-1/2, counted with multiplicity.

    Returns (lambda ascending, V n x k orthonormal[, info])."""
    op = NormalizedOperator(rowptr, col, val)
    n = op.n
    if not (1 <= k < n):
        raise ValueError("need 1 <= k < n")
    if m is None:
        m = min(n - 1, max(2 * k, 20))
    rng = np.random.default_rng(seed)
    eps = np.finfo(np.float64).eps
    tiny = eps * np.sqrt(n)

    X = np.zeros((n, 0))
    theta_x = np.zeros(0)
    cycles = 0
    phases = 0
    done = False
    converged = True

    while not done:
        nl = X.shape[1]
        room = n - nl                       # dimension of the deflated space
        if room <= 0:
            break
        if cycles >= maxiter:
            converged = nl >= k
            break
        cap = min(room, max(2, min(m, n) - nl))
        phases += 1
        cycles += 1

        # -- start vector: uniform(-1,1), orthogonal to the locked vectors
        while True:
            v = rng.uniform(-1.0, 1.0, size=n)
            _cgs2(v, [X])
            nv = np.linalg.norm(v)
            if nv > 1e-8 * np.sqrt(n):
                break
        V = np.zeros((n, cap + 1))
        V[:, 0] = v / nv
        T = np.zeros((cap, cap))
        j = 0                               # Lanczos vectors that have been multiplied by S

        while True:
            w = op(V[:, j])
            _, hv = _cgs2(w, [X, V[:, : j + 1]])
            T[j, j] = hv[j]                 # alpha_j
            beta = np.linalg.norm(w)
            j += 1
            breakdown = beta <= tiny

            th, Y = np.linalg.eigh(T[:j, :j])
            th, Y = th[::-1], Y[:, ::-1]    # descending theta
            rho = np.abs(beta * Y[j - 1, :])
            lead = 0
            while lead < j and rho[lead] <= tol:
                lead += 1

            if lead >= 1 or breakdown or j == room:
                if lead == 0:               # invariant subspace reached: every Ritz pair is exact
                    lead = j
                want = max(1, k - nl)
                nlock = min(lead, want)
                if nl >= k:
                    kth = np.sort(theta_x)[::-1][k - 1]
                    if th[0] <= kth + tol:
                        done = True         # a fresh deflated phase found nothing better
                newx = V[:, :j] @ Y[:, :nlock]
                X = np.hstack([X, newx])
                theta_x = np.concatenate([theta_x, th[:nlock]])
                if X.shape[1] >= n:
                    done = True
                break

            if j == cap:
                # thick restart: leading Ritz vectors + residual vector
                if cycles >= maxiter:
                    # out of cycles: hand back the best unconverged Ritz vectors of this phase
                    take = min(j, max(0, k - nl))
                    X = np.hstack([X, V[:, :j] @ Y[:, :take]])
                    theta_x = np.concatenate([theta_x, th[:take]])
                    converged = False
                    done = True
                    break
                cycles += 1
                keep = max(1, min(cap - 1, cap // 2))
                V[:, :keep] = V[:, :j] @ Y[:, :keep]
                V[:, keep] = w / beta
                coupling = beta * Y[j - 1, :keep]
                T[:, :] = 0.0
                T[np.arange(keep), np.arange(keep)] = th[:keep]
                T[keep, :keep] = coupling
                T[:keep, keep] = coupling
                j = keep
                continue

            V[:, j] = w / beta
            T[j, j - 1] = beta
            T[j - 1, j] = beta

    # -- Rayleigh-Ritz over everything locked (the Ritz-vector step of Algorithm 3)
    nl = X.shape[1]
    if nl == 0:
        raise RuntimeError("nothing converged")
    q, _ = np.linalg.qr(X)
    g = q.T @ op(q)
    g = 0.5 * (g + g.T)
    th, Y = np.linalg.eigh(g)
    th, Y = th[::-1], Y[:, ::-1]
    kk = min(k, nl)
    lam = 1.0 - th[:kk]
    vec = q @ Y[:, :kk]
    if nl < k:
        converged = False
    info = {"phases": phases, "cycles": cycles, "spmv": op.count, "locked": nl, "converged": converged}
    return (lam, vec, info) if return_info else (lam, vec)
