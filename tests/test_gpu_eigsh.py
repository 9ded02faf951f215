"""GPU parity of the whole hot path (sc_laplacian_eigsh through the C ABI) against the CPU oracle.

Bars (eigenvalue / residual / angle) are in tests/parity.py.  Inside a multiple eigenvalue any
orthonormal basis is correct, so subspaces are compared per separated cluster; when k cuts a cluster the
GPU vectors must lie in the oracle's cluster space."""
import math
import os

import numpy as np
import pytest

from oracle import dense, lanczos, components, compare
from paper_1802_04450_amd import workloads as wl
from parity import check_against_oracle

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1802_04450_amd import binding
    binding.lib()
    return binding


def solve(B, graph, k, tol, **kw):
    rp, c, v, n = graph
    drp, dc, dv = B.csr_to_device(rp, c, v)
    evals, evecs, code, stats = B.sc_laplacian_eigsh(drp, dc, dv, k, tol, **kw)
    return evals.cpu().numpy(), evecs.cpu().numpy().T.copy(), code, stats


CLOSED_FORM = [
    ("ring50", lambda: wl.ring(50), 5),
    ("path60", lambda: wl.path(60), 5),
    ("hypercube6", lambda: wl.hypercube(6), 7),
    ("complete12", lambda: wl.complete(12), 4),
    ("bipartite4x7", lambda: wl.complete_bipartite(4, 7), 3),
    ("union", lambda: wl.disjoint_union(wl.ring(9), wl.ring(14), wl.path(11), wl.random_weighted_connected(40, 80, 7),
                                        wl.complete(6)), 7),
    ("ring301", lambda: wl.ring(301), 9),
]


@pytest.mark.parametrize("name,make,k", CLOSED_FORM, ids=[c[0] for c in CLOSED_FORM])
def test_closed_form_graphs_match_dense_oracle(B, name, make, k):
    g = make()
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    lam, vec, code, stats = solve(B, g, k, 1e-10)
    assert code == B.SC_OK, stats
    check_against_oracle(g, k, lam, vec, lam_full[:k + 1], vec_full[:, :k])


@pytest.mark.parametrize("block", [1, 2, 4, 8, 16, 32])
def test_block_sizes_on_multiplicity_graph(B, block):
    # 6 components -> 6 zeros; then the rings' double eigenvalues
    g = wl.disjoint_union(*[wl.ring(20 + 3 * t) for t in range(6)])
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    k = 9
    lam, vec, code, stats = solve(B, g, k, 1e-10, block=block, m=max(60, k + 3 * block))
    assert code == B.SC_OK and stats["block"] == block
    check_against_oracle(g, k, lam, vec, lam_full[:k + 1], vec_full[:, :k])
    assert np.sum(np.abs(lam) < 1e-9) == 6


def test_config1_full_size(B):
    cfg = wl.CONFIGS[1]
    g, label, _ = wl.build_config_graph(cfg, device="cpu")
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    lam, vec, code, stats = solve(B, g, cfg.k, cfg.tol)
    assert code == B.SC_OK, stats
    out = check_against_oracle(g, cfg.k, lam, vec, lam_full[:cfg.k + 1], vec_full[:, :cfg.k],
                               cluster_basis=components.null_space(rp, c, v))
    assert np.max(np.abs(lam)) < 1e-9
    # also against the Lanczos oracle, and for more pairs than components (k = 12 > 8)
    lam_o, vec_o = lanczos.lanczos_smallest(rp, c, v, k=13, tol=1e-11, seed=3)
    lam2, vec2, code2, _ = solve(B, g, 12, cfg.tol)
    assert code2 == B.SC_OK
    check_against_oracle(g, 12, lam2, vec2, lam_o, vec_o)


def test_seed_independence_and_determinism(B):
    cfg = wl.reduced(wl.CONFIGS[1], n=1500, components=6, k=8)
    g, _, _ = wl.build_config_graph(cfg, device="cpu")
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    a = solve(B, g, 8, 1e-10, seed=1)
    b = solve(B, g, 8, 1e-10, seed=1)
    c2 = solve(B, g, 8, 1e-10, seed=2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])      # bitwise reproducible
    for out in (a, c2):
        check_against_oracle(g, 8, out[0], out[1], lam_full[:9], vec_full[:, :8])


REDUCED = [
    # (config id, n, components, k, m)   -- reduced instances of the large workloads, same recipe
    (2, 6000, 12, 12, 48),
    (3, 8000, 20, 10, 40),      # k < number of components: k cuts the null cluster
    (5, 6000, 30, 30, 96),
]


@pytest.mark.parametrize("cid,n,comps,k,m", REDUCED, ids=[f"cfg{r[0]}_n{r[1]}" for r in REDUCED])
def test_reduced_workloads_against_lanczos_and_component_oracles(B, cid, n, comps, k, m):
    cfg = wl.reduced(wl.CONFIGS[cid], n=n, components=comps, k=k, m=m)
    g, label, _ = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, nn = g
    ncomp, _ = components.component_labels(rp, c, v)
    lam_o, vec_o = lanczos.lanczos_smallest(rp, c, v, k=k + 1, tol=1e-10, m=max(m, 2 * (k + 1)), seed=11)
    lam, vec, code, stats = solve(B, g, k, cfg.tol, m=m)
    assert code == B.SC_OK, stats
    basis = components.null_space(rp, c, v) if k <= ncomp else None
    check_against_oracle(g, k, lam, vec, lam_o, vec_o, cluster_basis=basis)
    assert np.sum(np.abs(lam) < 1e-8) == min(k, ncomp)


def test_block32_on_reduced_large_k_workload(B):
    """The block size the library picks for the reorthogonalization-dominated workload (n >= 300,000 and k >= 1000:
    32 columns per step), end to end on a reduced instance of the same recipe, against the Lanczos oracle and the
    closed-form null space."""
    cfg = wl.reduced(wl.CONFIGS[5], n=12000, components=48, k=48, m=160)
    g, label, _ = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, nn = g
    ncomp, _ = components.component_labels(rp, c, v)
    k = cfg.k
    lam_o, vec_o = lanczos.lanczos_smallest(rp, c, v, k=k + 1, tol=1e-10, m=max(cfg.m, 2 * (k + 1)), seed=11)
    lam, vec, code, stats = solve(B, g, k, cfg.tol, m=cfg.m, block=32)
    assert code == B.SC_OK and stats["block"] == 32, stats
    basis = components.null_space(rp, c, v) if k <= ncomp else None
    check_against_oracle(g, k, lam, vec, lam_o, vec_o, cluster_basis=basis)
    assert np.sum(np.abs(lam) < 1e-8) == min(k, ncomp)


def test_reduced_blob_workload_3d(B):
    """Config-4 recipe at reduced size: anisotropic 3-D blobs, near-null ladder above the zeros."""
    cfg = wl.reduced(wl.CONFIGS[4], n=20000, components=6, k=6, m=60)
    g, label, _ = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, nn = g
    ncomp, _ = components.component_labels(rp, c, v)
    k = 6
    lam, vec, code, stats = solve(B, g, k, cfg.tol, m=cfg.m)
    assert code == B.SC_OK, stats
    lam_c, vec_c = components.smallest_eigenpairs(rp, c, v, k + 1, dense_limit=1500, tol=1e-10)
    check_against_oracle(g, k, lam, vec, lam_c, vec_c)


def test_maxiter_gives_not_converged_with_finite_output(B):
    g = wl.random_weighted_connected(3000, 9000, seed=9)
    lam, vec, code, stats = solve(B, g, 6, 1e-13, m=24, block=2, maxiter=1)
    assert code == B.SC_NOT_CONVERGED
    assert np.all(np.isfinite(lam)) and np.all(np.diff(lam) >= 0)
    assert compare.orthonormality_defect(vec) < 1e-9


def test_solver_rejects_bad_inputs_on_device(B):
    rp = np.array([0, 1, 1, 2, 3], dtype=np.int64)
    c = np.array([2, 0, 2], dtype=np.int32)
    v = np.array([1.0, 1.0, 1.0])
    drp, dc, dv = B.csr_to_device(rp, c, v)
    with pytest.raises(B.ScError) as e:
        B.sc_laplacian_eigsh(drp, dc, dv, 1, 1e-8, m=4, block=1)
    assert e.value.code == B.SC_EZERODEG
    bad = torch.tensor([2, 0, 9], dtype=torch.int32, device="cuda")
    with pytest.raises(B.ScError) as e:
        B.sc_laplacian_eigsh(drp, bad, dv, 1, 1e-8, m=4, block=1)
    assert e.value.code == B.SC_ECSR


def test_config2_full_size_bench_configuration(B):
    """The benchmark workload at full size (n = 100,000, k = 100, m = 200, tol 1e-8) in the launch
    configuration bench.py times.  Reference: the closed-form null space of the 100 components (exact),
    eigenvalue 0 with multiplicity 100; residuals recomputed on the host."""
    cfg = wl.CONFIGS[2]
    g, label, _ = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, n = g
    ncomp, _ = components.component_labels(rp, c, v)
    assert ncomp == cfg.components
    lam, vec, code, stats = solve(B, g, cfg.k, cfg.tol, m=cfg.m)
    assert code == B.SC_OK, stats
    basis = components.null_space(rp, c, v)
    out = check_against_oracle(g, cfg.k, lam, vec, np.zeros(cfg.k), basis, cluster_basis=basis)
    assert np.max(compare.principal_angles(vec, basis)) <= 1e-5
    print("config2", stats, out)


def _interleaved_components_graph():
    parts = [wl.ring(30), wl.path(41), wl.random_weighted_connected(200, 500, 3), wl.hypercube(5), wl.complete(9),
             wl.random_weighted_connected(333, 900, 4)]
    g = wl.disjoint_union(*parts)
    perm = np.random.default_rng(12).permutation(g[3])
    return wl.relabel(g, perm), len(parts)


def test_internal_reordering_is_invisible(B):
    """The component pass renumbers nodes internally; outputs must be in the caller's numbering and agree with
    the run that uses the CSR as given."""
    g, ncomp = _interleaved_components_graph()
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    k = 9
    a = solve(B, g, k, 1e-10)
    b = solve(B, g, k, 1e-10, flags=B.SC_FLAG_NO_REORDER)
    assert a[3]["components"] == ncomp == components.component_labels(rp, c, v)[0]
    assert b[3]["components"] == 0
    for out in (a, b):
        assert out[2] == B.SC_OK
        check_against_oracle(g, k, out[0], out[1], lam_full[:k + 1], vec_full[:, :k])


def test_zero_weight_entries_do_not_connect(B):
    # two rings joined by one explicit zero-weight edge: still two components, two zero eigenvalues
    g = wl.disjoint_union(wl.ring(40), wl.ring(50))
    rp, c, v, n = g
    extra_u, extra_v = np.array([3]), np.array([60])
    rows = np.repeat(np.arange(n), np.diff(rp))
    g2 = wl.coo_to_csr(np.concatenate([rows, extra_u, extra_v]), np.concatenate([c.astype(np.int64), extra_v, extra_u]),
                       np.concatenate([v, [0.0, 0.0]]), n, sum_duplicates=False)
    lam, vec, code, stats = solve(B, g2, 3, 1e-10)
    assert code == B.SC_OK and stats["components"] == 2 == components.component_labels(*g2[:3])[0]
    lam_full, vec_full = dense.full_spectrum(*g2[:3])
    check_against_oracle(g2, 3, lam, vec, lam_full[:4], vec_full[:, :3])


@pytest.mark.parametrize("k", [4, 6, 9])
def test_component_nullspace_option(B, k):
    """Optional pre-pass: the closed-form null vectors of the components are locked first (k below, equal to
    and above the number of components)."""
    g, ncomp = _interleaved_components_graph()
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    lam, vec, code, stats = solve(B, g, k, 1e-10, flags=B.SC_FLAG_COMPONENT_NULLSPACE)
    assert code == B.SC_OK
    basis = components.null_space(rp, c, v) if k <= ncomp else None
    if k == ncomp:
        check_against_oracle(g, k, lam, vec, lam_full[:k + 1], vec_full[:, :k], cluster_basis=basis)
    else:
        check_against_oracle(g, k, lam, vec, lam_full[:k] if k < ncomp else lam_full[:k + 1],
                             vec_full[:, :k], cluster_basis=basis)
    assert np.sum(np.abs(lam) < 1e-12) == min(k, ncomp)


@pytest.mark.parametrize("flags", ["NO_START_FILTER", "FINAL_RR", "NO_START_FILTER|FINAL_RR"])
def test_option_flags_give_the_same_answer(B, flags):
    """The start-block filter and the final Rayleigh-Ritz step are accelerations/refinements: with either switched
    the other way the answer must meet the same bars (multiplicity graph and a reduced clustered workload)."""
    f = 0
    for name in flags.split("|"):
        f |= getattr(B, "SC_FLAG_" + name)
    g = wl.disjoint_union(*[wl.ring(20 + 3 * t) for t in range(6)])
    lam_full, vec_full = dense.full_spectrum(*g[:3])
    lam, vec, code, stats = solve(B, g, 9, 1e-10, m=60, flags=f)
    assert code == B.SC_OK
    if f & B.SC_FLAG_NO_START_FILTER:
        assert stats["filter_steps"] == 0
    check_against_oracle(g, 9, lam, vec, lam_full[:10], vec_full[:, :9])
    cfg = wl.reduced(wl.CONFIGS[2], n=6000, components=12)
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    k = 12
    lam, vec, code, stats = solve(B, g, k, 1e-8, flags=f)
    assert code == B.SC_OK
    ncomp, _ = components.component_labels(*g[:3])
    assert ncomp >= k              # the reduced workload keeps its clusters disconnected: k exact zeros
    basis = components.null_space(*g[:3])
    assert np.max(np.abs(lam)) <= 1e-8
    assert np.max(compare.residual_norms(*g[:3], lam, vec)) <= 1e-6
    assert np.max(compare.containment_defect(vec, basis)) <= 1e-5
    assert compare.orthonormality_defect(vec) <= 1e-9


def test_start_filter_is_used_on_clustered_workload(B):
    """On a union of components (eigenvalue 0 with multiplicity > block size) the re-injection blocks are filtered and
    the phases after the first need only a few Lanczos steps."""
    cfg = wl.reduced(wl.CONFIGS[2], n=6000, components=24)
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    lam, vec, code, with_filter = solve(B, g, 24, 1e-8, block=4)
    assert code == B.SC_OK and with_filter["filter_steps"] > 0
    lam2, vec2, code2, without = solve(B, g, 24, 1e-8, block=4, flags=B.SC_FLAG_NO_START_FILTER)
    assert code2 == B.SC_OK and without["filter_steps"] == 0
    assert with_filter["block_steps"] < without["block_steps"]
    assert np.max(np.abs(lam)) <= 1e-8 and np.max(np.abs(lam2)) <= 1e-8


def test_block_products_through_the_resident_form(B, monkeypatch):
    """Where every diagonal block of the renumbered operator has work items of the LDS-resident filter, the single
    products of the block steps run as a one-step recurrence of that form.  Both ways of multiplying must pass the
    parity bars against the component oracle and agree with each other to the tolerance."""
    cfg = wl.reduced(wl.CONFIGS[5], n=16000, components=64)
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, n = g
    basis = components.null_space(rp, c, v)
    k = basis.shape[1]
    assert 64 <= k <= 80
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")   # small graph: the cost model would leave the form out
    results = []
    for off in (False, True):
        if off:
            monkeypatch.setenv("SCEIG_NO_RESIDENT_PRODUCT", "1")
        before = B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS)
        lam, vec, code, stats = solve(B, g, k, 1e-9, block=16)
        assert code == B.SC_OK and stats["block_steps"] > 0, stats
        assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) > before       # the resident plan was in use
        assert np.max(np.abs(lam)) <= 1e-9
        assert compare.residual_norms(rp, c, v, lam, vec).max() <= 1e-8
        assert np.max(compare.containment_defect(vec, basis)) <= 1e-7
        assert compare.orthonormality_defect(vec) <= 1e-10
        results.append(lam)
    assert np.max(np.abs(results[0] - results[1])) <= 1e-9


def test_single_precision_filter_steps_change_nothing_that_is_returned(B, monkeypatch):
    """The one-launch start-block filter runs all steps but a double-precision tail in single precision.  The filter only
    prepares a start block, so the returned pairs must meet the same bars with and without it, and the phases must
    not need more block steps than a couple (the later steps damp what the rounding of the earlier ones adds)."""
    cfg = wl.reduced(wl.CONFIGS[5], n=16000, components=64)
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, n = g
    basis = components.null_space(rp, c, v)
    k = basis.shape[1]
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")   # small graph: the cost model would leave the form out
    runs = []
    for tail in (None, "1000"):
        if tail:
            monkeypatch.setenv("SCEIG_FILTER_FP64_TAIL", tail)   # every step in double precision
        lam, vec, code, stats = solve(B, g, k, 1e-9, block=32, m=k + 128)
        assert code == B.SC_OK and stats["filter_steps"] > 0, stats
        assert np.max(np.abs(lam)) <= 1e-9
        assert compare.residual_norms(rp, c, v, lam, vec).max() <= 1e-8
        assert np.max(compare.containment_defect(vec, basis)) <= 1e-7
        assert compare.orthonormality_defect(vec) <= 1e-10
        runs.append(stats)
    assert runs[0]["block_steps"] <= runs[1]["block_steps"] + 2, (runs[0], runs[1])


def test_filter_interval_with_a_wrong_spectrum_bottom(B, monkeypatch):
    """The start-block filters damp [estimate of the spectrum's bottom, a] instead of [-1, a].  Isolated eigenvalues at
    the bottom (the -1 of a bipartite component, here K_{3,4}: 7 of 12,007 nodes) are found by the first unfiltered
    steps; what those steps underestimate is the edge of a bulk, by a bounded amount that the margin covers.  This
    test makes the estimate wrong on purpose (-0.05 and +0.2 where the spectrum ends at -0.3 and -1): the filters then
    amplify what lies below it, the solver sees Ritz values below its estimate and lowers it, and all k null vectors
    still come back within the parity bars - a wrong estimate costs block steps, never correctness."""
    cfg = wl.reduced(wl.CONFIGS[2], n=12000, components=40)
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    g = wl.disjoint_union(g, wl.complete_bipartite(3, 4))
    rp, c, v, n = g
    ncomp, _ = components.component_labels(rp, c, v)
    assert ncomp == 41
    basis = components.null_space(rp, c, v)
    lam0, vec0, code0, stats0 = solve(B, g, 41, 1e-8, block=16)
    assert code0 == B.SC_OK
    for forced in ("-0.05", "0.2"):
        monkeypatch.setenv("SCEIG_SPECTRUM_BOTTOM", forced)
        lam, vec, code, stats = solve(B, g, 41, 1e-8, block=16)
        assert code == B.SC_OK and stats["filter_steps"] > 0, stats
        assert np.max(np.abs(lam)) <= 1e-8
        assert compare.residual_norms(rp, c, v, lam, vec).max() <= 1e-7
        assert np.max(compare.containment_defect(vec, basis)) <= 1e-6
        assert compare.orthonormality_defect(vec) <= 1e-10


def test_release_cache_between_calls(B):
    """Workspace blocks are kept between calls; giving them back must not change any later result."""
    g = wl.disjoint_union(*[wl.ring(20 + 3 * t) for t in range(6)])
    lam1, vec1, code1, _ = solve(B, g, 9, 1e-10, m=60, seed=5)
    lam2, vec2, code2, _ = solve(B, g, 9, 1e-10, m=60, seed=5)        # served from the kept blocks
    assert B.sc_release_cache() == B.SC_OK
    lam3, vec3, code3, _ = solve(B, g, 9, 1e-10, m=60, seed=5)        # fresh allocations again
    assert code1 == code2 == code3 == B.SC_OK
    assert np.array_equal(lam1, lam2) and np.array_equal(lam1, lam3)
    assert np.array_equal(vec1, vec2) and np.array_equal(vec1, vec3)


@pytest.mark.parametrize("extra", [0, "FINAL_RR"])
def test_random_walk_vectors_of_the_papers_laplacian(B, extra):
    """SC_FLAG_RANDOM_WALK_VECTORS: eigenvectors of L_n = D^-1 L (Section II Steps 2-3).  Checked against the
    definition (L_n u = lambda u entry by entry), D-orthonormality, constancy on components for lambda = 0, and
    against the symmetric-form output of the same solve scaled by the oracle."""
    from oracle import laplacian
    parts = [wl.ring(9), wl.path(14), wl.random_weighted_connected(30, 60, 5), wl.complete(5), wl.ring(21)]
    g = wl.disjoint_union(*parts)
    g = wl.relabel(g, np.random.default_rng(8).permutation(g[3]))
    rp, c, v, n = g
    k = 8
    f = B.SC_FLAG_RANDOM_WALK_VECTORS | (getattr(B, "SC_FLAG_" + extra) if extra else 0)
    lam, u, code, _ = solve(B, g, k, 1e-10, flags=f, seed=3)
    lam_v, vec, code_v, _ = solve(B, g, k, 1e-10, flags=f & ~B.SC_FLAG_RANDOM_WALK_VECTORS, seed=3)
    assert code == code_v == B.SC_OK
    assert np.array_equal(lam, lam_v)
    assert np.max(np.abs(u - laplacian.random_walk_vectors(rp, c, v, vec))) <= 1e-14      # one scaling by s = d^-1/2
    lam_full, _ = dense.full_spectrum(rp, c, v)
    assert np.max(np.abs(lam - lam_full[:k])) <= 1e-8
    assert np.max(np.abs(laplacian.apply_random_walk_laplacian(rp, c, v, u) - u * lam[None, :])) <= 1e-6
    d = laplacian.degrees(rp, c, v)
    assert np.max(np.abs(u.T @ (d[:, None] * u) - np.eye(k))) <= 1e-9
    ncomp, label = components.component_labels(rp, c, v)
    for t in range(ncomp):
        for comp in range(ncomp):
            assert np.ptp(u[label == comp, t]) <= 1e-8


def _random_family(seed):
    """Seeded small graphs that exercise the solver's decisions: connected graphs without a gap, unions of
    components of uneven size (multiplicity above, at and below the block size), k below / at / above the
    multiplicity, tight and generous basis budgets."""
    rng = np.random.default_rng(1000 + seed)
    kind = seed % 4
    if kind == 0:                                   # one connected graph, dense spectrum
        n = int(rng.integers(80, 400))
        g = wl.random_weighted_connected(n, int(rng.integers(2, 6)) * n, seed)
        k = int(rng.integers(2, 12))
    elif kind == 1:                                 # many small components, k cuts the null cluster
        parts = [wl.random_weighted_connected(int(rng.integers(6, 40)), 60, seed * 31 + t) for t in range(int(rng.integers(5, 30)))]
        g = wl.disjoint_union(*parts)
        k = int(rng.integers(2, len(parts)))
    elif kind == 2:                                 # k beyond the number of components
        parts = [wl.ring(int(rng.integers(8, 30))) if t % 2 else wl.random_weighted_connected(int(rng.integers(10, 50)), 90, seed * 17 + t)
                 for t in range(int(rng.integers(3, 12)))]
        g = wl.disjoint_union(*parts)
        k = len(parts) + int(rng.integers(1, 6))
    else:                                           # k equal to the multiplicity, strongly uneven sizes
        sizes = [int(s) for s in rng.integers(5, 120, size=int(rng.integers(4, 20)))]
        parts = [wl.random_weighted_connected(s, 3 * s, seed * 13 + t) for t, s in enumerate(sizes)]
        g = wl.disjoint_union(*parts)
        k = len(parts)
    g = wl.relabel(g, rng.permutation(g[3]))
    n = g[3]
    k = max(1, min(k, n - 2))
    m = int(min(n, k + rng.choice([8, 24, 60]) + 3))
    return g, k, m


@pytest.mark.parametrize("seed", range(int(os.environ.get("SCEIG_RANDOM_CASES", "24"))))
def test_random_graph_families_against_dense_oracle(B, seed):
    g, k, m = _random_family(seed)
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    try:
        lam, vec, code, stats = solve(B, g, k, 1e-10, m=m, seed=seed)
    except B.ScError as e:                          # the budget can be too tight for any block size: a domain error
        assert e.args[0] == B.SC_EDOMAIN and k + 3 > m
        return
    assert code == B.SC_OK, stats
    check_against_oracle(g, k, lam, vec, lam_full[:k + 1], vec_full[:, :k])


def test_row_normalized_embedding(B):
    """SC_FLAG_ROW_NORMALIZE: the rows of the output (the points k-means clusters, Section II Step 4) have unit norm and
    equal the rows of the plain output divided by their norm; on a union of components with k = their number the rows
    of one component coincide and rows of different components are orthogonal."""
    parts = [wl.ring(9), wl.path(14), wl.random_weighted_connected(30, 60, 5), wl.complete(5), wl.ring(21)]
    g = wl.disjoint_union(*parts)
    g = wl.relabel(g, np.random.default_rng(9).permutation(g[3]))
    rp, c, v, n = g
    k = len(parts)
    _, vec, code, _ = solve(B, g, k, 1e-10, seed=3)
    for f in (B.SC_FLAG_ROW_NORMALIZE, B.SC_FLAG_ROW_NORMALIZE | B.SC_FLAG_RANDOM_WALK_VECTORS):
        _, emb, code2, _ = solve(B, g, k, 1e-10, seed=3, flags=f)
        assert code == code2 == B.SC_OK
        assert np.max(np.abs(np.linalg.norm(emb, axis=1) - 1.0)) <= 1e-14
        assert np.max(np.abs(emb - vec / np.linalg.norm(vec, axis=1, keepdims=True))) <= 1e-13
        _, label = components.component_labels(rp, c, v)
        gram = emb @ emb.T
        same = label[:, None] == label[None, :]
        assert np.max(np.abs(gram[same] - 1.0)) <= 1e-7 and np.max(np.abs(gram[~same])) <= 1e-7


def test_workspace_estimate_covers_what_a_solve_allocates(B):
    """sc_workspace_bytes against the device memory that actually leaves the free pool during a solve (the library
    keeps its blocks cached afterwards, so the drop in free memory is what the solve took)."""
    cfg = wl.reduced(wl.CONFIGS[2], n=60000, components=60, k=60)
    g, _, _ = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, n = g
    drp, dc, dv = B.csr_to_device(rp, c, v)
    B.sc_release_cache()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    evals, evecs, code, stats = B.sc_laplacian_eigsh(drp, dc, dv, cfg.k, 1e-8, m=cfg.m)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    taken = free0 - free1 - evals.numel() * 8 - evecs.numel() * 8      # the outputs are torch's, allocated in between
    est = B.sc_workspace_bytes(n, int(rp[-1]), cfg.k, m=cfg.m)
    assert code == B.SC_OK
    assert 0.8 * taken <= est <= 1.5 * taken + (32 << 20), (taken, est)
    B.sc_release_cache()
