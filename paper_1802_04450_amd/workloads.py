"""Seeded synthetic inputs: similarity graphs in CSR (int64 rowptr, int32 col, fp64 val).

This module only *builds inputs*.  It holds none of the eigensolver's arithmetic (no degrees,
no Laplacian, no Lanczos) and is shared by the tests of the CPU oracle and of the HIP library.

Two families:

* closed-form graphs (ring, path, complete, complete bipartite, hypercube, disjoint unions) whose
  normalized-Laplacian spectra are known analytically;
* the five Gaussian-mixture / blob kNN workloads: points drawn from a seeded mixture, an exact
  Euclidean k-nearest-neighbour graph symmetrized by union ("either direction", the kNN graph
  of the paper's Section IV-A list of graph types), weights exp(-dist^2 / (2 sigma^2)) with sigma
  the median of all directed kNN distances (the exponential-decay similarity of Section IV-A with
  the sign and square restored), self loops and exactly-zero weights dropped.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import numpy as np

CSR = Tuple[np.ndarray, np.ndarray, np.ndarray, int]  # rowptr(int64), col(int32), val(f64), n

BASE_SEED = 1802044500


# --------------------------------------------------------------------------------------------
# CSR assembly helpers (pure index bookkeeping)
# --------------------------------------------------------------------------------------------
def coo_to_csr(rows, cols, vals, n: int, sum_duplicates: bool = True) -> CSR:
    """Sort COO triples by (row, col) and compress the row indices."""
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    vals = np.asarray(vals, dtype=np.float64)
    key = rows * n + cols
    order = np.argsort(key, kind="stable")
    key, vals = key[order], vals[order]
    if sum_duplicates and key.size:
        uniq, start = np.unique(key, return_index=True)
        vals = np.add.reduceat(vals, start)
        key = uniq
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(np.bincount(rows, minlength=n))
    return rowptr, cols.astype(np.int32), vals, int(n)


def symmetric_from_edges(u, v, w, n: int) -> CSR:
    """Undirected edge list -> symmetric CSR (both directions stored once each)."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    w = np.asarray(w, dtype=np.float64)
    return coo_to_csr(np.concatenate([u, v]), np.concatenate([v, u]), np.concatenate([w, w]), n,
                      sum_duplicates=False)


def disjoint_union(*graphs: CSR) -> CSR:
    """Block-diagonal union; node ids of graph t are shifted by the sizes before it."""
    rp, cs, vs, off, nnz = [np.zeros(1, dtype=np.int64)], [], [], 0, 0
    for rowptr, col, val, n in graphs:
        rp.append(rowptr[1:] + nnz)
        cs.append(col.astype(np.int64) + off)
        vs.append(val)
        off += n
        nnz += int(rowptr[-1])
    return (np.concatenate(rp), np.concatenate(cs).astype(np.int32), np.concatenate(vs), off)


def relabel(graph: CSR, perm: np.ndarray) -> CSR:
    """Rename node i -> perm[i]."""
    rowptr, col, val, n = graph
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    return coo_to_csr(perm[rows], perm[col.astype(np.int64)], val, n, sum_duplicates=False)


# --------------------------------------------------------------------------------------------
# Closed-form graphs
# --------------------------------------------------------------------------------------------
def ring(n: int, weight: float = 1.0) -> CSR:
    i = np.arange(n, dtype=np.int64)
    return symmetric_from_edges(i, (i + 1) % n, np.full(n, weight), n)


def path(n: int, weight: float = 1.0) -> CSR:
    i = np.arange(n - 1, dtype=np.int64)
    return symmetric_from_edges(i, i + 1, np.full(n - 1, weight), n)


def complete(n: int, weight: float = 1.0) -> CSR:
    u, v = np.triu_indices(n, k=1)
    return symmetric_from_edges(u, v, np.full(u.size, weight), n)


def complete_bipartite(a: int, b: int, weight: float = 1.0) -> CSR:
    u = np.repeat(np.arange(a, dtype=np.int64), b)
    v = a + np.tile(np.arange(b, dtype=np.int64), a)
    return symmetric_from_edges(u, v, np.full(u.size, weight), a + b)


def hypercube(dim: int, weight: float = 1.0) -> CSR:
    n = 1 << dim
    i = np.arange(n, dtype=np.int64)
    us, vs = [], []
    for bit in range(dim):
        j = i ^ (1 << bit)
        keep = i < j
        us.append(i[keep])
        vs.append(j[keep])
    u, v = np.concatenate(us), np.concatenate(vs)
    return symmetric_from_edges(u, v, np.full(u.size, weight), n)


def random_weighted_connected(n: int, extra_edges: int, seed: int) -> CSR:
    """A ring (so the graph is connected) plus random chords, uniform(0.1, 1) weights."""
    rng = np.random.default_rng(seed)
    i = np.arange(n, dtype=np.int64)
    u = [i]
    v = [(i + 1) % n]
    a = rng.integers(0, n, size=extra_edges)
    b = rng.integers(0, n, size=extra_edges)
    keep = a != b
    u.append(a[keep])
    v.append(b[keep])
    u, v = np.concatenate(u), np.concatenate(v)
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    key = np.unique(lo * n + hi)
    lo, hi = key // n, key % n
    w = rng.uniform(0.1, 1.0, size=lo.size)
    return symmetric_from_edges(lo, hi, w, n)


# --------------------------------------------------------------------------------------------
# Mixture points
# --------------------------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class MixtureConfig:
    """One of the five benchmark workloads (sizes may be overridden for reduced instances)."""
    name: str
    n: int
    d: int
    components: int
    box: Tuple[float, float]
    std: Tuple[float, float]          # per-component std drawn uniform in [lo, hi]
    weights: str                      # "equal" | "dirichlet5"
    k_nn: int
    k: int                            # eigenpairs wanted
    m: int                            # Krylov basis budget (0: library default)
    tol: float
    anisotropic: bool = False
    seed: int = BASE_SEED


CONFIGS = {
    1: MixtureConfig("cfg1_tiny", 2_000, 16, 8, (-10.0, 10.0), (1.0, 1.0), "equal", 10, 8, 0, 1e-10,
                     seed=BASE_SEED + 1),
    2: MixtureConfig("cfg2_100k", 100_000, 32, 100, (-20.0, 20.0), (0.5, 1.5), "dirichlet5", 20, 100, 200,
                     1e-8, seed=BASE_SEED + 2),
    3: MixtureConfig("cfg3_1m", 1_000_000, 64, 1_000, (-20.0, 20.0), (0.5, 1.5), "dirichlet5", 16, 500,
                     1_000, 1e-8, seed=BASE_SEED + 3),
    4: MixtureConfig("cfg4_blobs3d", 4_000_000, 3, 200, (0.0, 1000.0), (0.2, 2.0), "equal", 32, 200, 400,
                     1e-7, anisotropic=True, seed=BASE_SEED + 4),
    5: MixtureConfig("cfg5_largek", 500_000, 128, 2_000, (-30.0, 30.0), (1.0, 1.0), "equal", 10, 2_000,
                     4_000, 1e-7, seed=BASE_SEED + 5),
}


def reduced(cfg: MixtureConfig, n: int, components: int, k: Optional[int] = None,
            m: Optional[int] = None) -> MixtureConfig:
    """Same recipe at a smaller size (same points-per-component order of magnitude)."""
    k = components if k is None else k
    return dataclasses.replace(cfg, name=f"{cfg.name}_n{n}", n=n, components=components, k=k,
                               m=(2 * k if m is None else m))


def mixture_points(cfg: MixtureConfig) -> Tuple[np.ndarray, np.ndarray]:
    """Draw the points of a workload.  Returns (X fp64 n x d, component label per point).

    Points are left in iid order (not grouped by component)."""
    rng = np.random.default_rng(cfg.seed)
    c, d, n = cfg.components, cfg.d, cfg.n
    centers = rng.uniform(cfg.box[0], cfg.box[1], size=(c, d))
    if cfg.weights == "equal":
        p = np.full(c, 1.0 / c)
    elif cfg.weights == "dirichlet5":
        p = rng.dirichlet(np.full(c, 5.0))
    else:
        raise ValueError(cfg.weights)
    label = rng.choice(c, size=n, p=p)
    if cfg.anisotropic:
        # per blob: a random rotation (Q of a Gaussian matrix) and per-axis stds
        rot = np.empty((c, d, d))
        for t in range(c):
            q, r = np.linalg.qr(rng.standard_normal((d, d)))
            rot[t] = q * np.sign(np.diag(r))
        axis_std = rng.uniform(cfg.std[0], cfg.std[1], size=(c, d))
        g = rng.standard_normal((n, d)) * axis_std[label]
        x = centers[label] + np.einsum("nj,nij->ni", g, rot[label])
    else:
        std = rng.uniform(cfg.std[0], cfg.std[1], size=c)
        x = centers[label] + std[label, None] * rng.standard_normal((n, d))
    return x, label


# --------------------------------------------------------------------------------------------
# Exact kNN (excluding self), three engines chosen by shape
# --------------------------------------------------------------------------------------------
def _knn_tree(x: np.ndarray, k_nn: int):
    from scipy.spatial import cKDTree
    tree = cKDTree(x)
    dist, idx = tree.query(x, k=k_nn + 1, workers=-1)
    # drop self (first hit; with duplicate points self may not be first, so mask explicitly)
    n = x.shape[0]
    self_pos = np.argmax(idx == np.arange(n)[:, None], axis=1)
    has_self = (idx == np.arange(n)[:, None]).any(axis=1)
    self_pos = np.where(has_self, self_pos, k_nn)
    keep = np.ones_like(idx, dtype=bool)
    keep[np.arange(n), self_pos] = False
    return idx[keep].reshape(n, k_nn), dist[keep].reshape(n, k_nn)


def _knn_brute_torch(x: np.ndarray, k_nn: int, device: str, block: int = 4096):
    """Blocked brute force: candidate selection from |x|^2+|y|^2-2xy, distances recomputed
    from coordinate differences in fp64 for the selected pairs."""
    import torch
    n, d = x.shape
    dev = torch.device(device)
    sel_dtype = torch.float64
    xt = torch.from_numpy(x).to(dev, sel_dtype)
    sq = (xt * xt).sum(1)
    idx_out = np.empty((n, k_nn), dtype=np.int64)
    dist_out = np.empty((n, k_nn), dtype=np.float64)
    cand = min(n - 1, k_nn + 4)  # a few spare candidates; re-ranked exactly below
    import sys
    import time
    last = time.time()
    for r0 in range(0, n, block):
        if time.time() - last > 30.0:   # long builds say that they are alive
            print(f"[workloads] kNN rows {r0}/{n}", file=sys.stderr, flush=True)
            last = time.time()
        r1 = min(n, r0 + block)
        g = xt[r0:r1] @ xt.T
        d2 = sq[r0:r1, None] + sq[None, :] - 2.0 * g
        d2[torch.arange(r1 - r0, device=dev), torch.arange(r0, r1, device=dev)] = float("inf")
        _, ci = torch.topk(d2, cand, dim=1, largest=False)
        diff = xt[ci] - xt[r0:r1, None, :]
        exact = torch.sqrt((diff * diff).sum(2))
        order = torch.argsort(exact, dim=1, stable=True)[:, :k_nn]
        idx_out[r0:r1] = torch.gather(ci, 1, order).cpu().numpy()
        dist_out[r0:r1] = torch.gather(exact, 1, order).cpu().numpy()
    return idx_out, dist_out


def knn(x: np.ndarray, k_nn: int, device: Optional[str] = None):
    """Exact Euclidean k nearest neighbours excluding the point itself."""
    n, d = x.shape
    if d <= 8:
        return _knn_tree(x, k_nn)
    if device is None:
        import torch
        device = "cuda" if torch.cuda.is_available() else "cpu"
    return _knn_brute_torch(x, k_nn, device)


def knn_gaussian_graph(x: np.ndarray, k_nn: int, device: Optional[str] = None) -> Tuple[CSR, float]:
    """Union-symmetrized kNN graph with Gaussian weights.  Returns (CSR, sigma)."""
    import sys
    import time
    n = x.shape[0]
    big = n * k_nn >= 20_000_000

    def note(msg):   # long builds say that they are alive
        if big:
            print(f"[workloads] {msg} ({time.time() - t_start:.0f}s)", file=sys.stderr, flush=True)

    t_start = time.time()
    idx, dist = knn(x, k_nn, device)
    note("kNN done")
    sigma = float(np.median(dist))
    u = np.repeat(np.arange(n, dtype=np.int64), k_nn)
    v = idx.reshape(-1).astype(np.int64)
    dd = dist.reshape(-1)
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    key = lo * n + hi
    key, first = np.unique(key, return_index=True)       # union: one undirected edge per pair
    note("union done")
    dd = dd[first]
    w = np.exp(-(dd * dd) / (2.0 * sigma * sigma))
    keep = (w > 0.0) & ((key // n) != (key % n))           # drop underflowed weights / self loops
    key, w = key[keep], w[keep]
    lo, hi = key // n, key % n
    touched = np.zeros(n, dtype=bool)
    touched[lo] = True
    touched[hi] = True
    if not touched.all():
        # nodes whose every weight underflowed are isolated: remove them (Section IV-B assumes
        # positive degrees, "otherwise the isolated nodes can be removed from the graph")
        newid = np.cumsum(touched) - 1
        lo, hi, n = newid[lo], newid[hi], int(touched.sum())
    graph = symmetric_from_edges(lo, hi, w, n)
    note("CSR done")
    return graph, sigma


def build_config_graph(cfg: MixtureConfig, device: Optional[str] = None):
    """Points -> kNN graph for a workload.  Returns (CSR, labels, sigma)."""
    x, label = mixture_points(cfg)
    graph, sigma = knn_gaussian_graph(x, cfg.k_nn, device)
    return graph, label, sigma


# ---- second workload family: connected graphs without the exact multiplicities of the mixture workloads -------------
def stochastic_block_model(n: int, blocks: int, p: float, q: float, seed: int) -> Tuple[CSR, np.ndarray]:
    """Unit-weight stochastic block model in the style of the paper's Syn200 (Section V-A): `blocks` equal groups,
    an edge with probability p inside a group and q between groups.  Returns (graph, group of every node).
    Edge counts are drawn per group pair (binomial) and the pairs uniformly inside it, so the cost is O(edges)."""
    rng = np.random.default_rng(seed)
    size = n // blocks
    assert size * blocks == n and size >= 2
    group = np.repeat(np.arange(blocks), size)
    us, vs = [], []
    # inside the groups: every group has size*(size-1)/2 pairs
    pairs_in = size * (size - 1) // 2
    iu, iv = np.triu_indices(size, 1)
    for b in range(blocks):
        pick = np.flatnonzero(rng.random(pairs_in) < p)
        us.append(b * size + iu[pick])
        vs.append(b * size + iv[pick])
    # between the groups: geometric skipping over the n*(n-1)/2 pairs would be exact; at the small q used here a
    # binomial number of uniformly drawn cross pairs (duplicates dropped) differs from it by O(q) relative
    cross_pairs = n * (n - 1) // 2 - blocks * pairs_in
    m_cross = int(rng.binomial(cross_pairs, q))
    a = rng.integers(0, n, size=int(m_cross * 1.02) + 16)
    b2 = rng.integers(0, n, size=a.size)
    keep = group[a] != group[b2]
    a, b2 = a[keep][:m_cross], b2[keep][:m_cross]
    us.append(np.minimum(a, b2))
    vs.append(np.maximum(a, b2))
    u = np.concatenate(us)
    v = np.concatenate(vs)
    key = np.unique(u.astype(np.int64) * n + v)
    u, v = key // n, key % n
    return symmetric_from_edges(u, v, np.ones(u.size), n), group


def preferential_attachment(n: int, edges_per_node: float, seed: int) -> CSR:
    """Unit-weight graph with a power-law degree tail (preferential attachment): node t > m0 attaches floor or ceil of
    `edges_per_node` edges to earlier nodes drawn in proportion to their degree.  Connected by construction; hubs of
    degree ~ sqrt(n).  The shape of the paper's DBLP co-authorship graph (Table "Datasets": 317,080 nodes,
    1,049,866 edges) is n = 317080, edges_per_node = 3.311."""
    rng = np.random.default_rng(seed)
    lo = int(math.floor(edges_per_node))
    frac = edges_per_node - lo
    m0 = lo + 2
    # the multiset of edge endpoints; drawing a uniform element of it is drawing a node in proportion to its degree
    cap = int(2 * (edges_per_node + 1) * n) + 4 * m0 * m0
    ends = np.empty(cap, dtype=np.int64)
    us, vs = [], []
    fill = 0
    for a in range(m0):              # start from a small complete graph
        for b in range(a + 1, m0):
            us.append(a)
            vs.append(b)
            ends[fill] = a
            ends[fill + 1] = b
            fill += 2
    u_arr = np.empty(int((edges_per_node + 1) * n) + 8, dtype=np.int64)
    v_arr = np.empty_like(u_arr)
    ne = len(us)
    u_arr[:ne] = us
    v_arr[:ne] = vs
    extra = rng.random(n) < frac
    for t in range(m0, n):
        m = lo + (1 if extra[t] else 0)
        targets = np.unique(ends[rng.integers(0, fill, size=m)])
        k = targets.size
        u_arr[ne:ne + k] = targets
        v_arr[ne:ne + k] = t
        ne += k
        ends[fill:fill + k] = targets
        ends[fill + k:fill + 2 * k] = t
        fill += 2 * k
    return symmetric_from_edges(u_arr[:ne], v_arr[:ne], np.ones(ne), n)


# Shapes of the paper's own graph datasets (Table "Datasets"); the graphs are synthetic stand-ins of that shape.
# Syn200: the printed p = 0.3, q = 0.01 give ~2.3 M expected edges at n = 20,000 and 200 groups, the table says
# 773,388; q = 0.0024 matches the table's count and is what is used here.
SECOND_WORKLOADS = {
    "syn200": dict(kind="sbm", n=20_000, blocks=200, p=0.3, q=0.0024, k=200, tol=1e-8, seed=BASE_SEED + 11),
    # its wanted eigenvalues sit at the edge of a dense bulk (spacing ~1e-5): the basis budget is 3k, not 2k
    "dblp_like": dict(kind="pa", n=317_080, edges_per_node=3.311, k=500, m=1500, tol=1e-8, seed=BASE_SEED + 12),
    "fb_like": dict(kind="sbm", n=4_040, blocks=10, p=0.1, q=0.0006, k=10, tol=1e-8, seed=BASE_SEED + 13),
}


def build_second_workload(name: str, n: Optional[int] = None, blocks: Optional[int] = None):
    """(graph, spec) of one of SECOND_WORKLOADS, optionally at a reduced size of the same recipe."""
    spec = dict(SECOND_WORKLOADS[name])
    if n is not None:
        spec["n"] = n
    if blocks is not None:
        spec["blocks"] = blocks
        spec["k"] = blocks
    if spec["kind"] == "sbm":
        g, _ = stochastic_block_model(spec["n"], spec["blocks"], spec["p"], spec["q"], spec["seed"])
    else:
        g = preferential_attachment(spec["n"], spec["edges_per_node"], spec["seed"])
    return g, spec


# ---- point sets for the k-means step -------------------------------------------------------------------------------
def gaussian_blobs(n: int, d: int, k: int, seed: int, spread: float = 0.15) -> np.ndarray:
    """n points in d dimensions around k standard-normal centres (labels uniform), isotropic noise of std `spread`."""
    rng = np.random.default_rng(seed)
    cen = rng.normal(size=(max(k, 1), d))
    lab = rng.integers(0, max(k, 1), size=n)
    return cen[lab] + spread * rng.normal(size=(n, d))


def embedding_like(n: int, k: int, seed: int, noise: float = 1e-3) -> np.ndarray:
    """Rows of an orthonormal n x k matrix that is constant on k groups up to `noise`, scaled to unit length: the shape
    of the row-normalised spectral embedding of a graph with k clusters (Section II Steps 3-4)."""
    rng = np.random.default_rng(seed)
    lab = rng.integers(0, k, size=n)
    rot = np.linalg.qr(rng.normal(size=(k, k)))[0]
    q, _ = np.linalg.qr(rot[lab] + noise * rng.normal(size=(n, k)))
    return q / np.linalg.norm(q, axis=1, keepdims=True)


def voxel_neighbour_pairs(n: int, radius2: int = 5, side: Optional[int] = None):
    """Pair list of the shape of the paper's DTI input (Section V-A: 142,541 voxels, 3,992,290 pairs within 4 mm on a
    2 mm grid): the first n cells of a side^3 grid in x-fastest order, every pair of cells whose integer offset has
    squared length <= radius2 listed once (u < v).  radius2 = 5 gives 28 pairs per interior cell."""
    if side is None:
        side = int(math.ceil(n ** (1.0 / 3.0)))
    idx = np.arange(n, dtype=np.int64)
    ix, iy, iz = idx % side, (idx // side) % side, idx // (side * side)
    us, vs = [], []
    r = int(math.isqrt(radius2))
    for dz in range(0, r + 1):
        for dy in range(-r, r + 1):
            for dx in range(-r, r + 1):
                if dx * dx + dy * dy + dz * dz > radius2 or (dz, dy, dx) <= (0, 0, 0):
                    continue
                ok = (ix + dx >= 0) & (ix + dx < side) & (iy + dy >= 0) & (iy + dy < side) & (iz + dz < side)
                j = idx + dx + dy * side + dz * side * side
                ok &= j < n
                us.append(idx[ok])
                vs.append(j[ok])
    return np.concatenate(us).astype(np.int32), np.concatenate(vs).astype(np.int32)


def connectivity_profiles(n: int, d: int, seed: int, side: Optional[int] = None) -> np.ndarray:
    """n x d non-negative rows that vary smoothly over the voxel grid (a few smooth spatial modes per coordinate plus
    noise): the shape of the DTI connectivity profiles (d = 90 regions)."""
    rng = np.random.default_rng(seed)
    if side is None:
        side = int(math.ceil(n ** (1.0 / 3.0)))
    idx = np.arange(n)
    pos = np.stack([idx % side, (idx // side) % side, idx // (side * side)], axis=1) / side
    freq = rng.uniform(0.5, 3.0, size=(3, d))
    phase = rng.uniform(0, 2 * np.pi, size=d)
    return np.abs(np.sin(2 * np.pi * pos @ freq + phase) + 0.3 * rng.normal(size=(n, d)))


def describe(graph: CSR) -> dict:
    rowptr, col, val, n = graph
    deg = np.diff(rowptr)
    return {"n": int(n), "nnz": int(rowptr[-1]), "deg_min": int(deg.min()), "deg_med": float(np.median(deg)),
            "deg_max": int(deg.max())}
