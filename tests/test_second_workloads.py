"""Second workload family: connected graphs without exact multiplicities (stochastic block model in the style of the
paper's Syn200, preferential attachment with DBLP's node and edge counts; Section V-A, Table "Datasets").

CPU part: the generators give what they say.  GPU part: the eigensolver against the dense oracle at sizes the oracle
finishes in seconds, the sparse products on hub rows, and (opt-in, SCEIG_FULLSIZE=1) Syn200 at full size by residuals
and orthonormality."""

import numpy as np
import pytest

from oracle import components, dense, compare, laplacian
from paper_1802_04450_amd import workloads as wl
from parity import check_against_oracle


def _is_symmetric(g):
    from scipy.sparse import csr_matrix
    rp, c, v, n = g
    a = csr_matrix((v, c, rp), shape=(n, n))
    return (abs(a - a.T)).nnz == 0 and a.diagonal().sum() == 0.0


def test_sbm_generator_shape():
    g, group = wl.stochastic_block_model(2000, 20, 0.3, 0.01, 1)
    rp, c, v, n = g
    assert _is_symmetric(g) and np.all(v == 1.0)
    same = group[np.repeat(np.arange(n), np.diff(rp))] == group[c]
    pin = same.sum() / (20 * 100 * 99)          # directed pairs inside the groups
    pout = (~same).sum() / (n * (n - 1) - 20 * 100 * 99)
    assert abs(pin - 0.3) < 0.01 and abs(pout - 0.01) < 0.0005
    # same seed, same graph
    g2, _ = wl.stochastic_block_model(2000, 20, 0.3, 0.01, 1)
    assert np.array_equal(g2[1], c)


def test_syn200_has_the_table_size():
    g, spec = wl.build_second_workload("syn200")
    edges = int(g[0][-1]) // 2
    assert g[3] == 20000 and abs(edges - 773388) < 0.01 * 773388
    assert components.component_labels(*g[:3])[0] == 1


def test_preferential_attachment_shape():
    g = wl.preferential_attachment(20000, 3.311, 3)
    rp, c, v, n = g
    assert _is_symmetric(g)
    assert components.component_labels(rp, c, v)[0] == 1
    deg = np.diff(rp)
    assert abs(deg.sum() / 2 / n - 3.311) < 0.05
    assert deg.max() > 20 * np.median(deg)      # hubs
    # tail exponent of the degree distribution ~ 3 (slope of the complementary distribution ~ -2)
    ks = np.array([8, 16, 32, 64])
    ccdf = np.array([(deg >= k).mean() for k in ks])
    slope = np.polyfit(np.log(ks), np.log(ccdf), 1)[0]
    assert -2.6 < slope < -1.5, slope


gpu = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1802_04450_amd import binding
    binding.lib()
    return binding


def _solve(B, g, k, tol, **kw):
    rp, c, v, n = g
    drp, dc, dv = B.csr_to_device(rp, c, v)
    evals, evecs, code, stats = B.sc_laplacian_eigsh(drp, dc, dv, k, tol, **kw)
    return evals.cpu().numpy(), evecs.cpu().numpy().T.copy(), code, stats


@gpu
@pytest.mark.parametrize("name,make,k", [
    ("sbm3000", lambda: wl.stochastic_block_model(3000, 30, 0.3, 0.01, 5)[0], 30),
    ("sbm1200_k_cuts_the_bulk", lambda: wl.stochastic_block_model(1200, 12, 0.3, 0.01, 6)[0], 20),
    ("pa3000", lambda: wl.preferential_attachment(3000, 3.311, 6), 8),
    ("fb_like", lambda: wl.build_second_workload("fb_like")[0], 10),
])
def test_connected_graphs_match_dense_oracle(B, name, make, k):
    g = make()
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    assert lam_full[1] > 1e-3                   # connected: the zero eigenvalue is simple
    lam, vec, code, stats = _solve(B, g, k, 1e-9)
    assert code == B.SC_OK, stats
    check_against_oracle(g, k, lam, vec, lam_full[:k + 1], vec_full[:, :k])


@gpu
@pytest.mark.parametrize("b", [1, 4, 16])
def test_products_on_power_law_rows(B, b):
    """Hub rows of degree ~ sqrt(n) next to rows of degree 1-3: every row-to-lane mapping of the products."""
    g = wl.preferential_attachment(40000, 3.311, 9)
    rp, c, v, n = g
    assert np.diff(rp).max() > 300
    drp, dc, dv = B.csr_to_device(rp, c, v)
    _, s = B.sc_degree_scaling(drp, dc, dv, want_degrees=False)
    x = np.random.default_rng(b).standard_normal((n, b))
    y = B.sc_spmm_normalized(drp, dc, dv, s, torch.as_tensor(x, device="cuda:0")).cpu().numpy()
    ref = laplacian.apply_s(rp, c, v, x)
    assert np.max(np.abs(y - ref)) <= 1e-13 * max(1.0, np.max(np.abs(ref)))


@gpu
def test_syn200_full_size(B):
    g, spec = wl.build_second_workload("syn200")
    rp, c, v, n = g
    lam, vec, code, stats = _solve(B, g, spec["k"], spec["tol"])
    assert code == B.SC_OK, stats
    res = compare.residual_norms(rp, c, v, lam, vec)
    assert res.max() <= 1e-6 and compare.orthonormality_defect(vec) <= 1e-9
    assert abs(lam[0]) < 1e-12 and lam[1] > 0.3 and np.all(np.diff(lam) >= -1e-12)
    print("syn200", stats["t_total"], res.max())
