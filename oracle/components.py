"""Exact spectrum through connected components.

W of a graph with components C_1..C_c is block diagonal, so the spectrum of the normalized
Laplacian is the multiset union of the component spectra.  Each connected component contributes
exactly one eigenvalue 0 with eigenvector D^1/2 1_C / sqrt(vol(C)), vol(C) the sum of the degrees
in C (the volume of Section II's Ncut definition).  Anything beyond the zeros is obtained per
component: dense eigendecomposition for small components, the Lanczos oracle for large ones.
"""
from __future__ import annotations

import numpy as np

from .laplacian import degrees
from . import dense as _dense
from . import lanczos as _lanczos


def component_labels(rowptr, col, val):
    """(number of components, label per node); explicit zero weights do not connect."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import connected_components
    n = rowptr.size - 1
    # copies: eliminate_zeros() rewrites the index arrays in place and must not touch the caller's CSR
    pattern = csr_matrix(((np.asarray(val) != 0.0).astype(np.int8), np.array(col, copy=True),
                          np.array(rowptr, copy=True)), shape=(n, n))
    pattern.eliminate_zeros()
    c, label = connected_components(pattern, directed=False)
    return int(c), label


def null_space(rowptr, col, val):
    """Orthonormal basis (n x c) of the eigenvalue-0 eigenspace, one column per component."""
    n = rowptr.size - 1
    c, label = component_labels(rowptr, col, val)
    d = degrees(rowptr, col, val)
    vol = np.bincount(label, weights=d, minlength=c)
    basis = np.zeros((n, c))
    basis[np.arange(n), label] = np.sqrt(d / vol[label])
    return basis


def sub_csr(rowptr, col, val, nodes: np.ndarray):
    """CSR of the subgraph induced by ``nodes`` (a union of whole components)."""
    n = rowptr.size - 1
    newid = np.full(n, -1, dtype=np.int64)
    newid[nodes] = np.arange(nodes.size)
    counts = np.diff(rowptr)[nodes]
    rp = np.zeros(nodes.size + 1, dtype=np.int64)
    rp[1:] = np.cumsum(counts)
    take = np.repeat(np.asarray(rowptr)[nodes], counts) + (np.arange(rp[-1]) - np.repeat(rp[:-1], counts))
    return rp, newid[col[take].astype(np.int64)].astype(np.int32), np.asarray(val)[take]


def smallest_eigenpairs(rowptr, col, val, k: int, dense_limit: int = 3000, tol: float = 1e-12):
    """(lambda ascending [k], V n x k) assembled component by component."""
    n = rowptr.size - 1
    c, label = component_labels(rowptr, col, val)
    if k <= c:
        basis = null_space(rowptr, col, val)
        return np.zeros(k), basis[:, :k]
    lams, owners, vecs = [], [], []
    for t in range(c):
        nodes = np.flatnonzero(label == t)
        rp, cc, vv = sub_csr(rowptr, col, val, nodes)
        kk = min(k, nodes.size)
        if nodes.size <= dense_limit:
            lam, vec = _dense.smallest_eigenpairs(rp, cc, vv, kk)
        else:
            kk = min(kk, k - c + 1)
            lam, vec = _lanczos.lanczos_smallest(rp, cc, vv, kk, tol, seed=t)
        lams.append(lam)
        owners.append(np.full(lam.size, t))
        vecs.append((nodes, vec))
    lam_all = np.concatenate(lams)
    own_all = np.concatenate(owners)
    idx_in = np.concatenate([np.arange(l.size) for l in lams])
    order = np.argsort(lam_all, kind="stable")[:k]
    out = np.zeros((n, k))
    for pos, o in enumerate(order):
        nodes, vec = vecs[own_all[o]]
        out[nodes, pos] = vec[:, idx_in[o]]
    return lam_all[order], out
