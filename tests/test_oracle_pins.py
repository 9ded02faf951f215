"""Pins for the CPU oracle: closed-form spectra, invariants, brute force and mutual agreement.

No value here comes from the HIP path.  Closed forms (normalized Laplacian L = I - D^-1/2 W D^-1/2):
  ring C_n (unit weights):        lambda_j = 1 - cos(2 pi j / n), j = 0..n-1
  path P_n:                       lambda_j = 1 - cos(pi j / (n-1)), eigenvector D^1/2 u, u_i = cos(pi j i/(n-1))
  complete K_n:                   {0, n/(n-1) x (n-1)}
  complete bipartite K_{a,b}:     {0, 1 x (n-2), 2}
  hypercube Q_d:                  2 i / d with multiplicity C(d, i)
  disjoint union:                 multiset union; c components -> c zeros with eigenvectors
                                  D^1/2 1_C / sqrt(vol C)   (vol as in Section II)
"""
import math

import numpy as np
import pytest

from oracle import laplacian, dense, lanczos, components, compare
from paper_1802_04450_amd import workloads as wl


def ring_spectrum(n):
    return np.sort(1.0 - np.cos(2.0 * np.pi * np.arange(n) / n))


def path_spectrum(n):
    return np.sort(1.0 - np.cos(np.pi * np.arange(n) / (n - 1)))


def hypercube_spectrum(d):
    out = []
    for i in range(d + 1):
        out += [2.0 * i / d] * math.comb(d, i)
    return np.array(sorted(out))


# ------------------------------------------------------------------ operator / definitions
def test_degrees_and_operator_by_hand():
    # triangle 0-1 (w=1), 1-2 (w=2), 0-2 (w=3): d = (4, 3, 5)
    g = wl.symmetric_from_edges([0, 1, 0], [1, 2, 2], [1.0, 2.0, 3.0], 3)
    rp, c, v, n = g
    assert np.allclose(laplacian.degrees(rp, c, v), [4.0, 3.0, 5.0])
    s = laplacian.inv_sqrt_degrees(rp, c, v)
    assert np.allclose(s, [0.5, 1 / math.sqrt(3), 1 / math.sqrt(5)])
    x = np.array([1.0, -2.0, 0.5])
    w = np.array([[0, 1, 3], [1, 0, 2], [3, 2, 0]], dtype=float)
    expect = s * (w @ (s * x))
    assert np.allclose(laplacian.apply_s(rp, c, v, x), expect, rtol=0, atol=1e-15)
    op = laplacian.NormalizedOperator(rp, c, v)
    assert np.allclose(op(x), expect, rtol=0, atol=1e-15)
    lap = laplacian.dense_laplacian(rp, c, v)
    assert np.allclose(lap, np.eye(3) - np.diag(s) @ w @ np.diag(s), atol=1e-15)
    # a transposed operand or a dropped scaling breaks symmetry / the unit diagonal
    assert np.allclose(lap, lap.T, atol=1e-15) and np.allclose(np.diag(lap), 1.0)


def test_operator_matches_dense_on_random_graph_and_blocks():
    rp, c, v, n = wl.random_weighted_connected(200, 600, seed=3)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((n, 5))
    sd = laplacian.dense_s(rp, c, v)
    assert np.allclose(laplacian.apply_s(rp, c, v, x), sd @ x, atol=1e-13)
    assert np.allclose(laplacian.NormalizedOperator(rp, c, v)(x), sd @ x, atol=1e-13)


def test_zero_degree_rejected():
    rp = np.array([0, 1, 1, 2], dtype=np.int64)  # node 1 has no entries
    c = np.array([2, 0], dtype=np.int32)
    v = np.array([1.0, 1.0])
    with pytest.raises(ValueError):
        laplacian.inv_sqrt_degrees(rp, c, v)


# ------------------------------------------------------------------ dense oracle vs closed forms
@pytest.mark.parametrize("n", [5, 12, 31])
def test_dense_ring(n):
    lam, _ = dense.full_spectrum(*wl.ring(n)[:3])
    assert np.allclose(lam, ring_spectrum(n), atol=1e-13)


@pytest.mark.parametrize("n", [2, 7, 40])
def test_dense_path_values_and_vectors(n):
    rp, c, v, _ = wl.path(n)
    lam, vec = dense.full_spectrum(rp, c, v)
    assert np.allclose(lam, path_spectrum(n), atol=1e-13)
    d = laplacian.degrees(rp, c, v)
    i = np.arange(n)
    for j in range(n):                      # all simple: per-vector check up to sign
        u = np.sqrt(d) * np.cos(np.pi * j * i / (n - 1))
        u /= np.linalg.norm(u)
        assert abs(abs(u @ vec[:, j]) - 1.0) < 1e-10


def test_dense_complete_and_bipartite_and_hypercube():
    lam, _ = dense.full_spectrum(*wl.complete(9)[:3])
    assert np.allclose(lam, [0.0] + [9.0 / 8.0] * 8, atol=1e-13)
    lam, _ = dense.full_spectrum(*wl.complete_bipartite(3, 5)[:3])
    assert np.allclose(lam, [0.0] + [1.0] * 6 + [2.0], atol=1e-13)
    lam, _ = dense.full_spectrum(*wl.hypercube(4)[:3])
    assert np.allclose(lam, hypercube_spectrum(4), atol=1e-13)


def test_dense_invariants_trace_frobenius_range_scaling_relabel():
    g = wl.random_weighted_connected(150, 500, seed=11)
    rp, c, v, n = g
    lam, vec = dense.full_spectrum(rp, c, v)
    assert lam.min() > -1e-13 and lam.max() < 2.0 + 1e-13
    assert abs(lam.sum() - n) < 1e-10                         # trace(L) = n without self loops
    d = laplacian.degrees(rp, c, v)
    rows = laplacian.row_index(rp)
    fro = n + np.sum(v * v / (d[rows] * d[c]))
    assert abs(np.sum(lam * lam) - fro) < 1e-9                 # ||L||_F^2
    assert compare.orthonormality_defect(vec) < 1e-12
    lam2, _ = dense.full_spectrum(rp, c, 37.5 * v)             # W -> cW leaves L unchanged
    assert np.allclose(lam, lam2, atol=1e-13)
    perm = np.random.default_rng(5).permutation(n)
    lam3, _ = dense.full_spectrum(*wl.relabel(g, perm)[:3])
    assert np.allclose(lam, lam3, atol=1e-12)


def test_dense_disjoint_union_null_space():
    g = wl.disjoint_union(wl.ring(7), wl.path(5), wl.complete(4), wl.random_weighted_connected(30, 60, 2))
    rp, c, v, n = g
    lam, vec = dense.smallest_eigenpairs(rp, c, v, 4)
    assert np.allclose(lam, 0.0, atol=1e-13)
    basis = components.null_space(rp, c, v)
    assert basis.shape == (n, 4)
    assert compare.orthonormality_defect(basis) < 1e-14
    assert np.max(compare.principal_angles(vec, basis)) < 1e-7
    # the closed-form vectors really are null vectors of L
    assert np.max(compare.residual_norms(rp, c, v, np.zeros(4), basis)) < 1e-14
    full, _ = dense.full_spectrum(rp, c, v)
    expect = np.sort(np.concatenate([ring_spectrum(7), path_spectrum(5), [0.0] + [4 / 3] * 3,
                                     dense.full_spectrum(*wl.random_weighted_connected(30, 60, 2)[:3])[0]]))
    assert np.allclose(full, expect, atol=1e-12)


# ------------------------------------------------------------------ Lanczos oracle
def _check_pairs(g, lam, vec, lam_true, tol_val=1e-9, tol_res=1e-7):
    rp, c, v, n = g
    assert np.allclose(lam, lam_true[: lam.size], atol=tol_val), (lam, lam_true[: lam.size])
    assert compare.orthonormality_defect(vec) < 1e-10
    assert np.max(compare.residual_norms(rp, c, v, lam, vec)) < tol_res


def test_lanczos_path_simple_spectrum():
    g = wl.path(60)
    lam, vec, info = lanczos.lanczos_smallest(*g[:3], k=5, tol=1e-10, seed=1, return_info=True)
    _check_pairs(g, lam, vec, path_spectrum(60))
    assert info["converged"]


def test_lanczos_ring_multiplicity_two():
    g = wl.ring(50)
    lam, vec = lanczos.lanczos_smallest(*g[:3], k=5, tol=1e-10, seed=2)
    _check_pairs(g, lam, vec, ring_spectrum(50))                # 0, then two double eigenvalues


def test_lanczos_hypercube_high_multiplicity():
    d = 6
    g = wl.hypercube(d)
    lam, vec = lanczos.lanczos_smallest(*g[:3], k=1 + d, tol=1e-10, seed=3)
    _check_pairs(g, lam, vec, hypercube_spectrum(d))            # 0 and 2/d with multiplicity d


def test_lanczos_complete_and_bipartite_breakdown_and_negative_end():
    g = wl.complete(12)
    lam, vec = lanczos.lanczos_smallest(*g[:3], k=4, tol=1e-10, seed=4)
    _check_pairs(g, lam, vec, np.array([0.0] + [12 / 11] * 11))
    g = wl.complete_bipartite(4, 7)
    lam, vec = lanczos.lanczos_smallest(*g[:3], k=3, tol=1e-10, seed=5)
    _check_pairs(g, lam, vec, np.array([0.0] + [1.0] * 9 + [2.0]))   # theta = -1 must not be picked


def test_lanczos_components_give_zeros_with_indicator_vectors():
    parts = [wl.ring(9), wl.ring(14), wl.path(11), wl.random_weighted_connected(40, 80, 7), wl.complete(6)]
    g = wl.disjoint_union(*parts)
    rp, c, v, n = g
    lam, vec = lanczos.lanczos_smallest(rp, c, v, k=5, tol=1e-10, seed=6)
    assert np.max(np.abs(lam)) < 1e-12
    basis = components.null_space(rp, c, v)
    assert np.max(compare.principal_angles(vec, basis)) < 1e-8
    # one more than the number of components: the sixth is the smallest nonzero of any part
    lam6, vec6 = lanczos.lanczos_smallest(rp, c, v, k=7, tol=1e-10, seed=6)
    full, _ = dense.full_spectrum(rp, c, v)
    _check_pairs(g, lam6, vec6, full)


def test_lanczos_matches_dense_on_mixture_graph_and_is_seed_independent():
    cfg = wl.reduced(wl.CONFIGS[1], n=600, components=5, k=8, m=24)
    g, label, _ = wl.build_config_graph(cfg, device="cpu")
    rp, c, v, n = g
    ncomp, _ = components.component_labels(rp, c, v)
    full, fvec = dense.full_spectrum(rp, c, v)
    assert np.sum(full < 1e-12) == ncomp
    for seed in (0, 1):
        lam, vec, info = lanczos.lanczos_smallest(rp, c, v, k=8, tol=1e-10, m=24, seed=seed, return_info=True)
        _check_pairs(g, lam, vec, full)
        assert info["converged"]
    # thick restarts were exercised (basis budget 24 is far below the steps needed)
    assert info["cycles"] > info["phases"]


def test_lanczos_maxiter_reports_not_converged():
    g = wl.random_weighted_connected(300, 900, seed=9)
    lam, vec, info = lanczos.lanczos_smallest(*g[:3], k=6, tol=1e-12, m=12, seed=0, maxiter=1, return_info=True)
    assert not info["converged"]


# ------------------------------------------------------------------ component oracle
def test_component_oracle_matches_dense_beyond_the_zeros():
    parts = [wl.ring(9), wl.path(11), wl.random_weighted_connected(40, 80, 7), wl.hypercube(3)]
    g = wl.disjoint_union(*parts)
    perm = np.random.default_rng(1).permutation(g[3])
    g = wl.relabel(g, perm)                                       # components interleaved
    rp, c, v, n = g
    full, _ = dense.full_spectrum(rp, c, v)
    for k in (3, 4, 9):
        lam, vec = components.smallest_eigenpairs(rp, c, v, k)
        assert np.allclose(lam, full[:k], atol=1e-12)
        assert compare.orthonormality_defect(vec) < 1e-10
        assert np.max(compare.residual_norms(rp, c, v, lam, vec)) < 1e-10
    lam, vec = components.smallest_eigenpairs(rp, c, v, 6, dense_limit=20)   # forces the Lanczos branch
    assert np.allclose(lam, full[:6], atol=1e-9)


def test_planted_mistake_is_caught_by_the_pins():
    """The pins are sharp enough: dropping the second scaling (S -> D^-1 W D^0 ... i.e. the
    random-walk matrix applied as if symmetric) or the shift lambda = 1 - theta changes the ring /
    path numbers by far more than the tolerances used above."""
    rp, c, v, n = wl.path(7)
    s = laplacian.inv_sqrt_degrees(rp, c, v)
    w = np.zeros((n, n))
    w[laplacian.row_index(rp), c] = v
    wrong = np.eye(n) - (s * s)[:, None] * w                       # D^-1 W: not symmetric
    lam_wrong = np.sort(np.linalg.eigvalsh(0.5 * (wrong + wrong.T)))
    assert np.max(np.abs(lam_wrong - path_spectrum(n))) > 1e-3


# ------------------------------------------------------------------ comparison utilities
def test_principal_angles_and_containment_known_values():
    e = np.eye(4)
    a = e[:, :2]
    t = 1e-6
    b = np.stack([e[:, 0], math.cos(t) * e[:, 1] + math.sin(t) * e[:, 2]], axis=1)
    ang = compare.principal_angles(a, b)
    assert abs(ang[-1] - t) < 1e-12 and ang[0] < 1e-12
    assert np.allclose(compare.containment_defect(b, e[:, :3]), 0.0, atol=1e-15)
    assert abs(compare.containment_defect(b, a)[1] - math.sin(t)) < 1e-15


def test_separated_clusters():
    lam = np.array([0.0, 0.0, 1e-12, 0.3, 0.3000001, 0.5])
    runs = compare.separated_clusters(lam, 5, r_sum=1e-9)
    assert runs == [(0, 3), (3, 5)]
    runs = compare.separated_clusters(lam, 4, r_sum=1e-9)          # k cuts the (0.3, 0.3000001) pair
    assert runs == [(0, 3)]


# ------------------------------------------------------------------ the tiny benchmark workload
def test_config1_full_size_three_oracles_agree():
    """n = 2000, 8 mixture components: 8 zero eigenvalues (union-find count), indicator null space,
    Lanczos oracle == dense definition == component oracle."""
    cfg = wl.CONFIGS[1]
    g, label, _ = wl.build_config_graph(cfg, device="cpu")
    rp, c, v, n = g
    ncomp, _ = components.component_labels(rp, c, v)
    assert ncomp == cfg.components == 8
    full, fvec = dense.full_spectrum(rp, c, v)
    assert np.sum(np.abs(full) < 1e-12) == 8 and full[8] > 0.05
    lam, vec, info = lanczos.lanczos_smallest(rp, c, v, k=8, tol=cfg.tol, seed=0, return_info=True)
    assert info["converged"] and np.max(np.abs(lam)) < 1e-12
    basis = components.null_space(rp, c, v)
    assert np.max(compare.principal_angles(vec, basis)) < 1e-7
    assert np.max(compare.principal_angles(fvec[:, :8], basis)) < 1e-7
    lam10, vec10 = lanczos.lanczos_smallest(rp, c, v, k=10, tol=cfg.tol, seed=1)
    assert np.allclose(lam10, full[:10], atol=1e-10)
    lamc, vecc = components.smallest_eigenpairs(rp, c, v, 10)
    assert np.allclose(lamc, full[:10], atol=1e-11)


def test_component_labels_leave_the_input_untouched_and_ignore_zero_weights():
    g = wl.disjoint_union(wl.ring(6), wl.ring(5))
    rp, c, v, n = g
    rows = np.repeat(np.arange(n), np.diff(rp))
    g2 = wl.coo_to_csr(np.concatenate([rows, [1], [8]]), np.concatenate([c.astype(np.int64), [8], [1]]),
                       np.concatenate([v, [0.0, 0.0]]), n, sum_duplicates=False)
    before = [a.copy() for a in g2[:3]]
    ncomp, label = components.component_labels(*g2[:3])
    assert ncomp == 2 and len(set(label[:6])) == 1 and len(set(label[6:])) == 1 and label[0] != label[6]
    for a, b in zip(before, g2[:3]):
        assert np.array_equal(a, b)


def test_random_walk_vectors_are_eigenvectors_of_the_papers_laplacian():
    """Section II Steps 2-3 work with L_n = D^-1 L.  u = D^-1/2 v must satisfy L_n u = lambda u with the same lambda,
    be D-orthonormal, and - the textbook reason for using L_n - be constant on every connected component for
    lambda = 0, so that the null vectors span the component indicators exactly."""
    parts = [wl.ring(9), wl.path(14), wl.random_weighted_connected(30, 60, 5), wl.complete(5)]
    g = wl.disjoint_union(*parts)
    g = wl.relabel(g, np.random.default_rng(8).permutation(g[3]))
    rp, c, v, n = g
    lam, vec = dense.full_spectrum(rp, c, v)
    u = laplacian.random_walk_vectors(rp, c, v, vec)
    lnu = laplacian.apply_random_walk_laplacian(rp, c, v, u)
    assert np.max(np.abs(lnu - u * lam[None, :])) < 1e-12
    d = laplacian.degrees(rp, c, v)
    assert np.max(np.abs(u.T @ (d[:, None] * u) - np.eye(n))) < 1e-12
    ncomp, label = components.component_labels(rp, c, v)
    assert ncomp == 4 and np.all(np.abs(lam[:4]) < 1e-13)
    for t in range(4):                      # every null vector is constant on every component
        for comp in range(ncomp):
            vals = u[label == comp, t]
            assert np.ptp(vals) < 1e-12
    # the span of the null vectors is the span of the component indicators
    ind = np.stack([(label == comp).astype(float) for comp in range(ncomp)], axis=1)
    assert np.max(compare.containment_defect(ind / np.linalg.norm(ind, axis=0), np.linalg.qr(u[:, :4])[0])) < 1e-12
    # hand value: on a connected graph the null vector is the constant 1/sqrt(vol)
    rp1, c1, v1, n1 = wl.random_weighted_connected(12, 20, 2)
    lam1, vec1 = dense.full_spectrum(rp1, c1, v1)
    u1 = laplacian.random_walk_vectors(rp1, c1, v1, vec1[:, 0])
    assert np.allclose(np.abs(u1), 1.0 / np.sqrt(laplacian.degrees(rp1, c1, v1).sum()), atol=1e-13)


def test_chebyshev_filter_closed_form_on_eigenvectors():
    """An eigenvector of S with eigenvalue theta goes to T_d(t) v with t = (2 theta - a + 1)/(a + 1); T_d(t) =
    cos(d arccos t) inside [-1, 1] and cosh(d arccosh t) above 1 - the closed forms, not the recurrence."""
    from oracle import blockops
    g = wl.disjoint_union(wl.ring(11), wl.random_weighted_connected(25, 50, 4), wl.path(9))
    rp, c, v, n = g
    lam, vec = dense.full_spectrum(rp, c, v)
    theta = 1.0 - lam
    a, d = 0.35, 9
    y = blockops.chebyshev_filter(rp, c, v, vec, a, d)
    t = (2.0 * theta - a + 1.0) / (a + 1.0)
    inside = np.abs(t) <= 1.0
    factor = np.where(inside, np.cos(d * np.arccos(np.clip(t, -1, 1))), np.cosh(d * np.arccosh(np.maximum(t, 1.0))))
    assert inside.any() and (~inside).any()
    assert np.max(np.abs(y - vec * factor[None, :]) / np.maximum(1.0, np.abs(factor))[None, :]) < 1e-11
    assert np.all(np.abs(factor[inside]) <= 1.0 + 1e-12) and np.all(factor[~inside] > 1.0)
    # degree 1 and 2 by hand: g(S) x and 2 g(S)^2 x - x
    x = np.random.default_rng(1).standard_normal((n, 3))
    gs = (2.0 * laplacian.dense_s(rp, c, v) - (a - 1.0) * np.eye(n)) / (a + 1.0)
    assert np.max(np.abs(blockops.chebyshev_filter(rp, c, v, x, a, 1) - gs @ x)) < 1e-13
    assert np.max(np.abs(blockops.chebyshev_filter(rp, c, v, x, a, 2) - (2.0 * gs @ (gs @ x) - x))) < 1e-12


def test_kmeans_oracle_pins():
    """Algorithms 4-5 against what the mathematics fixes: hand-computed tiny cases, exact recovery of far-apart
    groups with centres equal to the group means, monotone objective, the fixed-point conditions, and the sampling
    rule of the seeding on a case whose draws can be followed by hand."""
    from oracle import kmeans as km
    # the generator: values in [0, 1), reproducible, different per index and seed
    u = [km.uniform01(7, i) for i in range(1000)]
    assert all(0.0 <= t < 1.0 for t in u) and len(set(u)) == 1000 and u[3] == km.uniform01(7, 3) != km.uniform01(8, 3)
    assert abs(np.mean(u) - 0.5) < 0.03 and abs(np.var(u) - 1.0 / 12.0) < 0.01
    # four points on a line, centres started at the two left points: by hand
    x = np.array([[0.0], [1.0], [9.0], [10.0]])
    labels, cen, iters, hist, conv = km.lloyd(x, x[:2], 10)
    # it 1: centres 0,1 -> labels 0,1,1,1 (objective 0+0+64+81); centres 0, 20/3
    # it 2: point 1 is nearer to 0 (1 < 5.67) -> labels 0,0,1,1; centres 0.5, 9.5;  it 3: unchanged
    assert labels.tolist() == [0, 0, 1, 1] and np.allclose(cen[:, 0], [0.5, 9.5]) and conv and iters == 3
    assert np.allclose(hist, [145.0, 1.0 + (9 - 20 / 3) ** 2 + (10 - 20 / 3) ** 2, 1.0])
    # ties go to the first centre; an empty cluster keeps its centre
    lab, _ = km.assign(np.array([[1.0]]), np.array([[0.0], [2.0]]))
    assert lab.tolist() == [0]
    assert np.array_equal(km.update_centroids(x, np.array([0, 0, 0, 0]), np.array([[5.0], [7.0]])), [[5.0], [7.0]])
    # far-apart groups: exact recovery whatever the seed, centres are the group means, objective = within-group scatter
    rng = np.random.default_rng(3)
    means = 100.0 * np.eye(5)[:, :4] + 50.0
    truth = rng.integers(0, 5, size=400)
    pts = means[truth] + rng.standard_normal((400, 4))
    for seed in range(5):
        labels, cen, iters, hist, conv = km.kmeans(pts, 5, seed)
        assert conv and np.all(np.diff(hist) <= 1e-9)
        perm = {int(labels[np.flatnonzero(truth == g)[0]]): g for g in range(5)}
        assert len(perm) == 5 and all(perm[int(l)] == t for l, t in zip(labels, truth))
        for j, g in perm.items():
            assert np.allclose(cen[j], pts[truth == g].mean(axis=0), atol=1e-12)
        scatter = sum(((pts[truth == g] - pts[truth == g].mean(axis=0)) ** 2).sum() for g in range(5))
        assert abs(km.objective(pts, labels, cen) - scatter) < 1e-9 * scatter
        # fixed point: every point is at least as near to its own centre as to any other
        lab2, dist = km.assign(pts, cen)
        assert np.array_equal(lab2, labels)
    # seeding: k = n distinct points picks every point once (a chosen point has distance 0 and cannot be drawn again)
    idx = km.kmeanspp_indices(pts[:40], 40, 11)
    assert sorted(idx.tolist()) == list(range(40))
    # seeding by hand: points 0, 1, 3 on a line, seed chosen so that the first draw is point 0: the second point is
    # 1 with probability 1/10 and 3 with probability 9/10 (squared distances 1 and 9)
    line = np.array([[0.0], [1.0], [3.0]])
    counts = {1: 0, 2: 0}
    tried = 0
    for seed in range(4000):
        if int(km.uniform01(seed, 0) * 3) != 0:
            continue
        tried += 1
        second = int(km.kmeanspp_indices(line, 2, seed)[1])
        assert second == (1 if km.uniform01(seed, 1) * 10.0 < 1.0 else 2)
        counts[second] += 1
    assert tried > 1000 and abs(counts[2] / tried - 0.9) < 0.03


def test_similarity_oracle_pins():
    """Section IV-A measures and Algorithm 1: hand-computed values, the library's Pearson correlation, invariances that
    a dropped mean, a missing norm or a wrong sign would break, and the harness's own Gaussian kNN weights."""
    from oracle import similarity as sim
    # hand computed: x0 = (1,2,3), x1 = (2,4,6.5), x2 = (3,1,2)
    x = np.array([[1.0, 2.0, 3.0], [2.0, 4.0, 6.5], [3.0, 1.0, 2.0]])
    u, v = np.array([0, 0, 1]), np.array([1, 2, 2])
    # centred rows: (-1,0,1), (-13/6,-1/6,14/6), (1,-1,0); norms sqrt2, sqrt(366)/6, sqrt2
    cc = sim.edge_similarity(x, u, v, sim.CROSS_CORRELATION)
    np.testing.assert_allclose(cc, [(27 / 6) / (np.sqrt(2) * np.sqrt(366) / 6), -1 / 2,
                                    (-12 / 6) / (np.sqrt(366) / 6 * np.sqrt(2))], rtol=1e-14)
    cs = sim.edge_similarity(x, u, v, sim.COSINE)
    np.testing.assert_allclose(cs, [29.5 / np.sqrt(14 * 62.25), 11 / 14, 23 / np.sqrt(62.25 * 14)], rtol=1e-14)
    ed = sim.edge_similarity(x, u, v, sim.EXP_DECAY, sigma=2.0)
    np.testing.assert_allclose(ed, np.exp(-np.array([17.25, 6.0, 30.25]) / 8.0), rtol=1e-14)
    np.testing.assert_allclose(sim.row_means(x), [2.0, 25 / 6, 2.0], rtol=1e-15)
    np.testing.assert_allclose(sim.centered_norms(x), [np.sqrt(2), np.sqrt(366) / 6, np.sqrt(2)], rtol=1e-15)
    # library Pearson correlation; invariances
    rng = np.random.default_rng(0)
    x = rng.normal(size=(40, 90)) + rng.normal(size=(40, 1)) * 3
    u, v = np.triu_indices(40, 1)
    cc = sim.edge_similarity(x, u, v, sim.CROSS_CORRELATION)
    np.testing.assert_allclose(cc, np.corrcoef(x)[u, v], rtol=1e-12, atol=1e-14)
    shift, scale = rng.normal(size=(40, 1)) * 10, rng.uniform(0.5, 2.0, size=(40, 1))
    np.testing.assert_allclose(sim.edge_similarity(x * scale + shift, u, v, sim.CROSS_CORRELATION), cc, atol=1e-12)
    cs = sim.edge_similarity(x, u, v, sim.COSINE)
    np.testing.assert_allclose(sim.edge_similarity(x * scale, u, v, sim.COSINE), cs, atol=1e-13)
    assert np.max(np.abs(sim.edge_similarity(x + shift, u, v, sim.COSINE) - cs)) > 1e-3      # not shift invariant
    assert np.all(np.abs(cc) <= 1 + 1e-14) and np.all(np.abs(cs) <= 1 + 1e-14)
    np.testing.assert_allclose(sim.edge_similarity(x, u[:5], u[:5], sim.CROSS_CORRELATION), 1.0, rtol=1e-14)
    ed = sim.edge_similarity(x, u, v, sim.EXP_DECAY, sigma=7.0)
    assert np.all((ed > 0) & (ed < 1))
    np.testing.assert_allclose(sim.edge_similarity(x, v, u, sim.EXP_DECAY, sigma=7.0), ed, rtol=0)
    # larger sigma, larger similarity; orthogonal transformations leave it alone
    assert np.all(sim.edge_similarity(x, u, v, sim.EXP_DECAY, sigma=9.0) > ed)
    q = np.linalg.qr(rng.normal(size=(90, 90)))[0]
    np.testing.assert_allclose(sim.edge_similarity(x @ q, u, v, sim.EXP_DECAY, sigma=7.0), ed, rtol=1e-10)
    # the harness's Gaussian kNN graph (its own distance code) carries exactly these weights
    pts = rng.normal(size=(300, 5))
    (rp, c, val, n), sigma = wl.knn_gaussian_graph(pts, 6, device="cpu")
    rows = np.repeat(np.arange(n), np.diff(rp))
    np.testing.assert_allclose(sim.edge_similarity(pts, rows, c, sim.EXP_DECAY, sigma=sigma), val, rtol=1e-12)
    # COO semantics: duplicates add, symmetrization mirrors off-diagonal pairs only
    a = sim.coo_to_dense([0, 0, 2, 1], [1, 1, 2, 0], [1.0, 2.0, 5.0, 4.0], 3, symmetrize=True)
    np.testing.assert_array_equal(a, [[0, 7, 0], [7, 0, 0], [0, 0, 5]])
    a = sim.coo_to_dense([0, 0, 2, 1], [1, 1, 2, 0], [1.0, 2.0, 5.0, 4.0], 3, symmetrize=False)
    np.testing.assert_array_equal(a, [[0, 3, 0], [4, 0, 0], [0, 0, 5]])


def test_knn_oracle_pins():
    """Section III-A's k-nearest-neighbour graph: points on a line with known neighbours and the tie rule, the
    library's KD-tree on random points, and the union rule against a dense adjacency matrix."""
    from scipy.spatial import cKDTree
    from oracle import knn
    # points 0, 1, 2, 3, 10 on a line: neighbours by hand; equal distances go to the lower index
    x = np.array([[0.0], [1.0], [2.0], [3.0], [10.0]])
    idx, dist = knn.knn_bruteforce(x, 2)
    np.testing.assert_array_equal(idx, [[1, 2], [0, 2], [1, 3], [2, 1], [3, 2]])
    np.testing.assert_allclose(dist, [[1, 2], [1, 1], [1, 1], [1, 2], [7, 8]], rtol=0, atol=0)
    # random points in 5 dimensions against the library's exact KD-tree search (no ties in random data)
    rng = np.random.default_rng(11)
    x = rng.standard_normal((400, 5))
    idx, dist = knn.knn_bruteforce(x, 7)
    td, ti = cKDTree(x).query(x, k=8)
    np.testing.assert_array_equal(idx, ti[:, 1:])
    np.testing.assert_allclose(dist, td[:, 1:], rtol=1e-13)
    assert np.all(np.diff(dist, axis=1) >= 0) and np.all(idx != np.arange(400)[:, None])
    # union rule: dense OR of the directed relation, upper triangle
    adj = np.zeros((400, 400), dtype=bool)
    adj[np.repeat(np.arange(400), 7), idx.reshape(-1)] = True
    und = adj | adj.T
    eu, ev = np.nonzero(np.triu(und, 1))
    u, v, w = knn.knn_union_pairs(idx, dist)
    np.testing.assert_array_equal(u, eu)
    np.testing.assert_array_equal(v, ev)
    np.testing.assert_allclose(w, np.sqrt(((x[u] - x[v]) ** 2).sum(axis=1)), rtol=1e-13)
    assert len(u) > 400 * 7 / 2 and len(u) < 400 * 7          # some pairs are mutual, not all
    # Gaussian weights: the similarity oracle's exponential-decay measure on the same pairs
    from oracle import similarity as sim
    _, _, g = knn.knn_union_pairs(idx, dist, sigma=0.8)
    np.testing.assert_allclose(g, sim.edge_similarity(x, u, v, sim.EXP_DECAY, 0.8), rtol=1e-12)


def test_cgs2_block_and_rotate_pins():
    """oracle/blockops.cgs2_block (the reorthogonalization inside TakeStep, Section IV-B: classical Gram-Schmidt applied
    twice) and blockops.rotate (FindEigenvectors of Algorithm 3: Ritz vectors V Y) against values worked by hand, the
    identities the definitions fix, and planted mistakes."""
    from oracle import blockops
    # by hand, exact in binary up to the thirds: q1 = (1,2,2)/3, q2 = (2,1,-2)/3, q3 = (2,-2,1)/3 is the third direction
    q = np.array([[1.0, 2.0], [2.0, 1.0], [2.0, -2.0]]) / 3.0
    w = np.array([[3.0, 0.0], [0.0, 3.0], [0.0, 3.0]])
    w_out, h = blockops.cgs2_block(q, w)
    # q1.w1 = 1, q2.w1 = 2, q1.w2 = 4, q2.w2 = -1;  w1 - q1 - 2 q2 = 2 q3,  w2 - 4 q1 + q2 = -q3
    assert np.allclose(h, [[1.0, 4.0], [2.0, -1.0]], atol=1e-15)
    q3 = np.array([2.0, -2.0, 1.0]) / 3.0
    assert np.allclose(w_out, np.stack([2.0 * q3, -q3], axis=1), atol=1e-15)
    assert np.array_equal(w, [[3.0, 0.0], [0.0, 3.0], [0.0, 3.0]])          # the input block is not modified

    rng = np.random.default_rng(5)
    n, j, b = 60, 7, 3
    qo, _ = np.linalg.qr(rng.standard_normal((n, j)))
    wi = rng.standard_normal((n, b))
    wo, h = blockops.cgs2_block(qo, wi)
    assert np.max(np.abs(qo.T @ wo)) < 1e-14                              # orthogonal to every column of Q
    assert np.max(np.abs(h - qo.T @ wi)) < 1e-14                          # H = Q^T W for an orthonormal Q
    assert np.max(np.abs(wo + qo @ h - wi)) < 1e-14                       # W_in = Q H + W_out
    # a block already orthogonal to Q comes back unchanged with H = 0
    perp = wi - qo @ (qo.T @ wi)
    perp -= qo @ (qo.T @ perp)
    wo2, h2 = blockops.cgs2_block(qo, perp)
    assert np.max(np.abs(h2)) < 1e-15 and np.max(np.abs(wo2 - perp)) < 1e-15

    # "applied twice" is what the second pass is for: a block that lies in span(Q) up to 1e-10 loses ten digits to
    # cancellation in one pass (what is left along Q is rounding of the size 1e-16 |w| against |w_out| = 1e-10 |w|)
    small = rng.standard_normal((n, b))
    small -= qo @ (qo.T @ small)
    near = qo @ rng.standard_normal((j, b)) + 1e-10 * small
    wo3, h3 = blockops.cgs2_block(qo, near)
    def defect(x):
        return np.max(np.abs(qo.T @ x)) / np.min(np.linalg.norm(x, axis=0))
    once = near - qo @ (qo.T @ near)
    assert defect(wo3) < 1e-14 and defect(once) > 1e-9
    # and for a basis that is orthonormal only to 1e-6, H1 + H2 is the least-squares coefficient block to second order
    # (H1 alone is off in first order)
    qe = qo + 1e-6 * rng.standard_normal((n, j))
    wo4, h4 = blockops.cgs2_block(qe, wi)
    h_ls = np.linalg.lstsq(qe, wi, rcond=None)[0]
    assert np.max(np.abs(h4 - h_ls)) < 1e-9 and np.max(np.abs(qe.T @ wi - h_ls)) > 1e-7
    assert np.max(np.abs(qe.T @ wo4)) < 1e-9 and np.max(np.abs(qe.T @ (wi - qe @ (qe.T @ wi)))) > 1e-7

    # planted mistakes: second pass computed from the block as it came in; H1 returned alone
    def stale_second_pass(qm, wm):
        h1 = qm.T @ wm
        out = wm - qm @ h1
        h2_ = qm.T @ wm
        return out - qm @ h2_, h1 + h2_
    ws, hs = stale_second_pass(q, w)
    assert np.max(np.abs(hs - [[1.0, 4.0], [2.0, -1.0]])) > 0.5 and np.max(np.abs(q.T @ ws)) > 0.5
    assert np.max(np.abs((qe.T @ wi) - h_ls)) > 100 * np.max(np.abs(h4 - h_ls))

    # rotation, by hand: column t of V Y is sum_r V[:, r] Y[r, t]
    v = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    y = np.array([[1.0, -1.0, 0.5], [2.0, 0.0, -1.0]])
    assert np.array_equal(blockops.rotate(v, y), [[5.0, -1.0, -1.5], [11.0, -3.0, -2.5], [17.0, -5.0, -3.5]])
    assert np.array_equal(blockops.rotate(v, np.eye(2)), v)
    # an orthonormal basis rotated by the eigenvectors of its projected matrix gives Ritz vectors: orthonormal, and
    # X^T A X diagonal with the Ritz values
    a = rng.standard_normal((n, n))
    a = a + a.T
    tproj = qo.T @ a @ qo
    ritz, yv = np.linalg.eigh(tproj)
    x = blockops.rotate(qo, yv[:, -3:])
    assert np.max(np.abs(x.T @ x - np.eye(3))) < 1e-14
    assert np.max(np.abs(x.T @ a @ x - np.diag(ritz[-3:]))) < 1e-12
    # planted mistake: the transposed coefficient block (only possible when square) gives something else
    ysq = np.array([[1.0, -1.0], [2.0, 0.0]])
    assert np.max(np.abs(v @ ysq.T - blockops.rotate(v, ysq))) > 1.0
