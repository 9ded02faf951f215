"""GPU parity of the k-means step (Section IV-C, Algorithms 4 and 5) against the oracle, through the C ABI.

Labels and chosen seeds are integers decided by fp64 arithmetic: both sides decide in fp64, the kernel on the expanded
form |c|^2 - 2<v,c> and the oracle on the direct sum of squared differences.  The two may differ only where two
candidates are equal to rounding, so: every label / seed must be the oracle's, or a candidate that the oracle's own
numbers cannot tell from its choice (checked, and such points must be rare); centres agree to 1e-11 relative."""
import numpy as np
import pytest

from oracle import kmeans as okm
from paper_1802_04450_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1802_04450_amd import binding
    binding.lib()
    return binding


def _blobs(n, d, k, seed, spread=0.15):
    return wl.gaussian_blobs(n, d, k, seed, spread)


def _embedding_like(n, k, seed):
    return wl.embedding_like(n, k, seed)


def _dev(a, dtype=torch.float64):
    return torch.as_tensor(np.ascontiguousarray(a), dtype=dtype, device="cuda:0")


def _check_labels(x, cen_used, labels_gpu, labels_ref, dist_ref, max_ambiguous):
    """labels_gpu equals labels_ref except where the oracle's distances to the two labels agree to rounding."""
    diff = np.flatnonzero(labels_gpu != labels_ref)
    scale = float((x * x).sum(axis=1).max() + (cen_used * cen_used).sum(axis=1).max())
    for i in diff:
        assert abs(dist_ref[i, labels_gpu[i]] - dist_ref[i, labels_ref[i]]) <= 1e-12 * scale, (i, dist_ref[i])
    assert diff.size <= max_ambiguous, diff.size


CASES = [
    # n, d, k: several 64-row tiles / 64-centre tiles with ragged tails, d not a multiple of 4, k = 1, k = n
    ("blobs", 5003, 7, 5),
    ("blobs", 12345, 33, 70),
    ("blobs", 4097, 130, 257),
    ("embed", 20011, 100, 100),
    ("blobs", 300, 3, 1),
    ("blobs", 64, 2, 64),
    ("uniform", 6000, 6, 40),
]


def _points(kind, n, d, k, seed):
    if kind == "blobs":
        return _blobs(n, d, max(k, 1), seed)
    if kind == "embed":
        return _embedding_like(n, k, seed)
    return np.random.default_rng(seed).uniform(-1, 1, size=(n, d))


@pytest.mark.parametrize("kind,n,d,k", CASES)
def test_kmeanspp_matches_oracle(B, kind, n, d, k):
    x = _points(kind, n, d, k, seed=n + k)
    for seed in (1, 2):
        ref = okm.kmeanspp_indices(x, k, seed)
        chosen, cen = B.sc_kmeanspp(_dev(x), k, seed)
        got = chosen.cpu().numpy().astype(np.int64)
        if not np.array_equal(got, ref):
            # a draw may land within rounding of a boundary of the prefix sums: then the neighbouring point is as valid
            first = int(np.flatnonzero(got != ref)[0])
            assert first > 0
            d2 = okm.sq_distances_to(x, x[ref[0]])
            for j in ref[1:first]:
                d2 = np.minimum(d2, okm.sq_distances_to(x, x[j]))
            cs = np.cumsum(d2)
            r = okm.uniform01(seed, first) * cs[-1]
            lo, hi = sorted((int(got[first]), int(ref[first])))
            assert np.all(np.abs(cs[lo:hi] - r) <= 1e-12 * cs[-1]), (first, got[first], ref[first])
            pytest.skip("draw within rounding of a prefix-sum boundary; later draws legitimately differ")
        np.testing.assert_array_equal(cen.cpu().numpy(), x[ref])


@pytest.mark.parametrize("colmajor", [False, True])
@pytest.mark.parametrize("kind,n,d,k", CASES)
def test_lloyd_matches_oracle(B, kind, n, d, k, colmajor):
    x = _points(kind, n, d, k, seed=7 * n + k)
    init = x[okm.kmeanspp_indices(x, k, 3)]
    labels_ref, cen_ref, iters_ref, hist_ref, conv_ref = okm.lloyd(x, init, 60)
    pts = _dev(x.T) if colmajor else _dev(x)
    labels, cen, code, st = B.sc_kmeans_lloyd(pts, _dev(init), 60, colmajor=colmajor)
    lg = labels.cpu().numpy().astype(np.int64)
    # the labels of the last step were computed from the centres before the (skipped or last) update
    _, dist_ref = okm.assign(x, cen_ref if conv_ref else init)
    if conv_ref:
        _check_labels(x, cen_ref, lg, labels_ref, dist_ref, max_ambiguous=max(2, n // 2000))
        assert st["iterations"] == iters_ref and st["converged"] == 1 and code == 0
        np.testing.assert_allclose(cen.cpu().numpy(), cen_ref, rtol=1e-11, atol=1e-12)
        assert abs(st["objective"] - hist_ref[-1]) <= 1e-9 * max(1.0, hist_ref[-1])
    else:
        assert code == 1 and st["converged"] == 0 and st["iterations"] == 60
    assert lg.min() >= 0 and lg.max() < k


def test_one_lloyd_step_element_by_element(B):
    """One labelling step + one update from fixed centres: no iteration, so every label and centre is comparable."""
    n, d, k = 7001, 19, 37
    x = _blobs(n, d, k, 5, spread=0.6)
    init = x[np.random.default_rng(1).choice(n, k, replace=False)].copy()
    init[5] = 100.0  # a centre that attracts nobody keeps its place
    labels_ref, dist_ref = okm.assign(x, init)
    cen_ref = okm.update_centroids(x, labels_ref, init)
    labels, cen, code, st = B.sc_kmeans_lloyd(_dev(x), _dev(init), 1)
    assert code == 1 and st["iterations"] == 1 and st["last_changes"] == n
    _check_labels(x, init, labels.cpu().numpy().astype(np.int64), labels_ref, dist_ref, max_ambiguous=0)
    np.testing.assert_allclose(cen.cpu().numpy(), cen_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(cen.cpu().numpy()[5], init[5])


def test_kmeans_whole_and_bitwise_repeatable(B):
    n, d, k = 30011, 24, 24
    x = _embedding_like(n, k, 9)
    labels_ref, cen_ref, iters_ref, hist_ref, conv_ref = okm.kmeans(x, k, 42, 100)
    assert conv_ref
    out = [B.sc_kmeans(_dev(x), k, 42, 100) for _ in range(2)]
    (l0, c0, code0, st0), (l1, c1, _, _) = out
    assert torch.equal(l0, l1) and torch.equal(c0, c1)
    assert code0 == 0 and st0["iterations"] == iters_ref
    np.testing.assert_array_equal(l0.cpu().numpy(), labels_ref)
    np.testing.assert_allclose(c0.cpu().numpy(), cen_ref, rtol=1e-11, atol=1e-12)


def test_kmeans_on_eigensolver_output(B):
    """Steps 3 and 4 of Section II chained on the device: row-normalised eigenvectors of a graph with 6 components
    are clustered into exactly those components."""
    from oracle import components as ocomp
    from paper_1802_04450_amd import workloads as wl
    cfg = wl.reduced(wl.CONFIGS[2], n=6007, components=6, k=6)
    (rp, c, v, n), _, _ = wl.build_config_graph(cfg, device="cpu")
    drp, dc, dv = B.csr_to_device(rp, c, v)
    evals, evecs, code, _ = B.sc_laplacian_eigsh(drp, dc, dv, 6, 1e-10, flags=B.SC_FLAG_ROW_NORMALIZE)
    assert code == 0
    labels, cen, kcode, st = B.sc_kmeans(evecs, 6, 5, 100, colmajor=True)
    ncomp, comp = ocomp.component_labels(rp, c, v)
    assert ncomp == 6 and kcode == 0
    lg = labels.cpu().numpy()
    # Points of one component share their embedding row (to the solver's tolerance), so squared-distance sampling
    # draws every seed from a component that has none yet, and the clustering is the component partition up to the
    # names of the clusters.
    pairs = {(int(a), int(b)) for a, b in zip(comp, lg)}
    assert len(pairs) == 6 and len({p[0] for p in pairs}) == 6 and len({p[1] for p in pairs}) == 6
    assert st["objective"] <= 1e-12 * n


def test_kmeans_argument_errors(B):
    x = _dev(np.zeros((10, 3)))
    lib = B.lib()
    out_l = torch.empty(10, dtype=torch.int32, device="cuda:0")
    out_c = torch.empty((4, 3), dtype=torch.float64, device="cuda:0")
    assert lib.sc_kmeans(x.data_ptr(), 3, 0, 10, 3, 11, 0, 10, out_l.data_ptr(), out_c.data_ptr(), None, None) == B.SC_EDOMAIN
    assert lib.sc_kmeans(x.data_ptr(), 3, 0, 10, 3, 0, 0, 10, out_l.data_ptr(), out_c.data_ptr(), None, None) == B.SC_EDOMAIN
    assert lib.sc_kmeans(x.data_ptr(), 2, 0, 10, 3, 4, 0, 10, out_l.data_ptr(), out_c.data_ptr(), None, None) == B.SC_EDOMAIN
    assert lib.sc_kmeans(None, 3, 0, 10, 3, 4, 0, 10, out_l.data_ptr(), out_c.data_ptr(), None, None) == B.SC_EINVAL
    assert lib.sc_kmeans(x.data_ptr(), 3, 0, 10, 3, 4, 0, 0, out_l.data_ptr(), out_c.data_ptr(), None, None) == B.SC_EDOMAIN
    assert lib.sc_kmeans_lloyd(x.data_ptr(), 3, 0, 10, 3, 4, None, 5, out_l.data_ptr(), None, None) == B.SC_EINVAL
