"""k-nearest-neighbour similarity graph (Section III-A, the list of similarity graphs: two points are connected if
either is among the k most similar points of the other; here "most similar" = nearest in Euclidean distance, the
benchmark workloads' choice, with the Gaussian weight exp(-|x_i - x_j|^2 / (2 sigma^2)) of Section IV-A).

Plain numpy fp64, one query point at a time, the definition written out: all n - 1 distances, then the k smallest.
Equal distances are ordered by the neighbour's index, so the result is unique.

Test infrastructure only."""
from __future__ import annotations

import numpy as np


def knn_bruteforce(x: np.ndarray, k: int):
    """idx[i] = the k points nearest to x_i other than i itself, nearest first (ties: lower index first);
    dist[i] = their Euclidean distances."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    if not 1 <= k <= n - 1:
        raise ValueError("k must be in [1, n-1]")
    idx = np.empty((n, k), dtype=np.int64)
    dist = np.empty((n, k), dtype=np.float64)
    ids = np.arange(n)
    for i in range(n):
        diff = x - x[i]
        d2 = (diff * diff).sum(axis=1)
        d2[i] = np.inf                                   # the point itself is not its own neighbour
        order = np.lexsort((ids, d2))[:k]                # by distance, then by index
        idx[i] = order
        dist[i] = np.sqrt(d2[order])
    return idx, dist


def knn_union_pairs(idx: np.ndarray, dist: np.ndarray, sigma: float = 0.0):
    """The undirected edges of the kNN graph, each once as (u < v), sorted by (u, v): {i, j} is an edge if j is in
    i's list or i is in j's.  Value of an edge: its distance, or exp(-dist^2 / (2 sigma^2)) if sigma > 0."""
    n, k = idx.shape
    best = {}
    for i in range(n):
        for s in range(k):
            j = int(idx[i, s])
            if j < 0 or j == i:
                continue
            key = (i, j) if i < j else (j, i)
            if key not in best:
                best[key] = float(dist[i, s])
    keys = sorted(best)
    u = np.array([a for a, _ in keys], dtype=np.int64)
    v = np.array([b for _, b in keys], dtype=np.int64)
    d = np.array([best[key] for key in keys], dtype=np.float64)
    if sigma > 0.0:
        d = np.exp(-(d * d) / (2.0 * sigma * sigma))
    return u, v, d
