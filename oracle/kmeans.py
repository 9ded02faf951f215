"""k-means on the rows of the eigenvector matrix (Section II Step 4, Section IV-C, Algorithms 4 and 5).

Plain definitions in numpy fp64: k-means++ seeding as Algorithm 5 states it (first point uniform, then points drawn
with probability proportional to the squared distance to the nearest centre chosen so far), Lloyd iterations as
Algorithm 4 states them (distances, labels, centres, until no label changes).  Distances are the direct sums of
squared differences, not the expanded form the paper uses for BLAS.  The uniform numbers are passed in through a
counter-based generator that the GPU side implements too (splitmix64 finaliser of seed and draw index).

Test infrastructure only."""
from __future__ import annotations

import numpy as np

_MASK = (1 << 64) - 1


def _mix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK
    return x ^ (x >> 31)


def uniform01(seed: int, index: int) -> float:
    """The index-th uniform number in [0, 1) of stream `seed`: top 53 bits of mix64(mix64(seed) + index)."""
    h = _mix64((_mix64(seed & _MASK) + index) & _MASK)
    return (h >> 11) * (1.0 / 9007199254740992.0)


def sq_distances_to(x: np.ndarray, point: np.ndarray) -> np.ndarray:
    diff = x - point[None, :]
    return np.einsum("ij,ij->i", diff, diff)


def kmeanspp_indices(x: np.ndarray, k: int, seed: int) -> np.ndarray:
    """Algorithm 5.  Draw i uses uniform01(seed, i).  A point is chosen as the first index whose inclusive prefix sum
    of squared distances exceeds u * total; if none does (all remaining distances zero, or rounding at the top end)
    the last point is taken."""
    n = x.shape[0]
    first = min(int(uniform01(seed, 0) * n), n - 1)
    chosen = [first]
    dist2 = sq_distances_to(x, x[first])
    for i in range(1, k):
        cs = np.cumsum(dist2)
        r = uniform01(seed, i) * cs[-1]
        j = int(np.searchsorted(cs, r, side="right"))
        j = min(j, n - 1)
        chosen.append(j)
        dist2 = np.minimum(dist2, sq_distances_to(x, x[j]))
    return np.asarray(chosen, dtype=np.int64)


def assign(x: np.ndarray, centroids: np.ndarray):
    """Label of every point = index of the nearest centre (the first one on ties); also the squared distances."""
    n, k = x.shape[0], centroids.shape[0]
    dist = np.empty((n, k))
    for j in range(k):
        dist[:, j] = sq_distances_to(x, centroids[j])
    labels = np.argmin(dist, axis=1)
    return labels, dist


def update_centroids(x: np.ndarray, labels: np.ndarray, old: np.ndarray) -> np.ndarray:
    """Mean of the points of every cluster; a cluster without points keeps its centre."""
    new = old.copy()
    for j in range(old.shape[0]):
        members = np.flatnonzero(labels == j)
        if members.size:
            new[j] = x[members].sum(axis=0) / members.size
    return new


def lloyd(x: np.ndarray, centroids: np.ndarray, max_iter: int):
    """Algorithm 4 step 3.  Returns labels, centres, iterations done, objective history (sum of squared distances of
    the labelling of each iteration to the centres it was computed from) and whether it stopped because no label
    changed."""
    centroids = np.array(centroids, dtype=np.float64, copy=True)
    labels = np.full(x.shape[0], -1, dtype=np.int64)
    history = []
    converged = False
    iters = 0
    for _ in range(max_iter):
        new_labels, dist = assign(x, centroids)
        history.append(float(dist[np.arange(x.shape[0]), new_labels].sum()))
        changes = int(np.count_nonzero(new_labels != labels))
        labels = new_labels
        iters += 1
        if changes == 0:
            converged = True
            break
        centroids = update_centroids(x, labels, centroids)
    return labels, centroids, iters, history, converged


def kmeans(x: np.ndarray, k: int, seed: int, max_iter: int = 100):
    init = x[kmeanspp_indices(x, k, seed)]
    return lloyd(x, init, max_iter)


def objective(x: np.ndarray, labels: np.ndarray, centroids: np.ndarray) -> float:
    diff = x - centroids[labels]
    return float(np.einsum("ij,ij->", diff, diff))
