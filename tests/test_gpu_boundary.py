"""GPU tests of the boundary's optional pieces (include/sceig.h): the caller-provided workspace variant, the start
vector and guard options, and the symmetry / sign validation flag - all through the C ABI."""
import numpy as np
import pytest

from oracle import dense, components, compare
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


def _multiplicity_graph():
    return wl.disjoint_union(*[wl.ring(20 + 3 * t) for t in range(6)])


@pytest.mark.parametrize("case", ["rings_b4", "knn_b16", "knn_b16_nullspace", "knn_b2_noreorder", "misaligned"])
def test_workspace_variant_allocates_nothing_and_matches(B, case):
    """sc_laplacian_eigsh_ws inside a torch-owned buffer of exactly sc_workspace_bytes: bitwise the answer of
    sc_laplacian_eigsh, and the device's free memory does not move during the call."""
    if case == "rings_b4":
        g, k, tol, kw = _multiplicity_graph(), 9, 1e-10, dict(m=60, block=4)
    else:
        cfg = wl.reduced(wl.CONFIGS[2], n=30000, components=30, k=30)
        g, _, _ = wl.build_config_graph(cfg, device="cuda")
        k, tol = 30, 1e-8
        kw = {"knn_b16": dict(m=cfg.m), "knn_b16_nullspace": dict(m=cfg.m, flags=B.SC_FLAG_COMPONENT_NULLSPACE),
              "knn_b2_noreorder": dict(m=cfg.m, block=2, flags=B.SC_FLAG_NO_REORDER), "misaligned": dict(m=cfg.m)}[case]
    rp, c, v, n = g
    drp, dc, dv = B.csr_to_device(rp, c, v)
    ref_vals, ref_vecs, code0, st0 = B.sc_laplacian_eigsh(drp, dc, dv, k, tol, seed=3, **kw)
    need = B.sc_workspace_bytes(n, int(rp[-1]), k, m=kw.get("m", 0), block=kw.get("block", 0), flags=kw.get("flags", 0))
    shift = 8 if case == "misaligned" else 0
    buf = torch.empty(need + shift, dtype=torch.uint8, device="cuda")
    ws = buf[shift:]
    evals = torch.empty(k, dtype=torch.float64, device="cuda")
    evecs = torch.empty((k, n), dtype=torch.float64, device="cuda")
    B.sc_release_cache()
    # one call first: the library's pinned host blocks and the runtime's own lazily created state come into being
    B.sc_laplacian_eigsh(drp, dc, dv, k, tol, seed=3, workspace=ws, out=(evals, evecs), **kw)
    B.sc_release_cache()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    _, _, code, st = B.sc_laplacian_eigsh(drp, dc, dv, k, tol, seed=3, workspace=ws, out=(evals, evecs), **kw)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, (free0, free1)
    assert code == code0 == B.SC_OK
    assert torch.equal(evals, ref_vals) and torch.equal(evecs, ref_vecs)
    assert st["block_steps"] == st0["block_steps"] and st["spmv_cols"] == st0["spmv_cols"]
    # too small a buffer is refused before anything is computed
    evals.fill_(-7.0)
    with pytest.raises(B.ScError) as e:
        B.sc_laplacian_eigsh(drp, dc, dv, k, tol, seed=3, workspace=ws[: need // 2], out=(evals, evecs), **kw)
    assert e.value.code == B.SC_ENOMEM
    assert torch.all(evals == -7.0)


def test_start_vector_option(B):
    """opt->v0 leads the first start block.  The answer meets the same bars whatever it is; an exact eigenvector as
    start vector (the one direction a Krylov space can do nothing with) is handled; and it is really used: on a
    connected graph with block size 1 the exact null vector D^1/2 1 converges in the first inspection."""
    from oracle import laplacian
    g = _multiplicity_graph()
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    rng = np.random.default_rng(0)
    starts = {"random": rng.standard_normal(n), "ones": np.ones(n), "null vector": np.sqrt(laplacian.degrees(rp, c, v)),
              "unit": np.eye(n)[5]}
    for name, x0 in starts.items():
        v0 = torch.from_numpy(np.ascontiguousarray(x0)).cuda()
        for block in (1, 4):
            lam, vec, code, st = B.sc_laplacian_eigsh(drp, dc, dv, 9, 1e-10, m=60, block=block, v0=v0)
            assert code == B.SC_OK, (name, block)
            check_against_oracle(g, 9, lam.cpu().numpy(), vec.cpu().numpy().T.copy(), lam_full[:10], vec_full[:, :9])
    gc = wl.relabel(wl.random_weighted_connected(500, 1500, 3), np.random.default_rng(1).permutation(500))
    rp, c, v, n = gc
    drp, dc, dv = B.csr_to_device(rp, c, v)
    null = torch.from_numpy(np.sqrt(laplacian.degrees(rp, c, v))).cuda()
    kw = dict(m=40, block=1, flags=B.SC_FLAG_NO_VERIFY)
    lam1, vec1, code1, with_v0 = B.sc_laplacian_eigsh(drp, dc, dv, 1, 1e-10, v0=null, **kw)
    lam2, vec2, code2, without = B.sc_laplacian_eigsh(drp, dc, dv, 1, 1e-10, **kw)
    assert code1 == code2 == B.SC_OK
    assert abs(float(lam1[0])) < 1e-12 and abs(float(lam2[0])) < 1e-9
    assert with_v0["block_steps"] < without["block_steps"]
    assert with_v0["block_steps"] <= 4       # the first scheduled inspection


def test_guard_option(B):
    """opt->guard: k + guard pairs are converged and locked, the k leading ones returned (k = 7 cuts the rings' double
    eigenvalues; with guard the pairs beyond the cut are computed as well and then left out)."""
    rings = [wl.ring(30 + 2 * t) for t in range(5)]
    g = wl.disjoint_union(*rings)
    rp, c, v, n = g
    lam_full, vec_full = dense.full_spectrum(rp, c, v)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    for guard in (0, 3, 8):
        lam, vec, code, st = B.sc_laplacian_eigsh(drp, dc, dv, 7, 1e-10, m=80, block=4, guard=guard)
        assert code == B.SC_OK and lam.numel() == 7 and vec.shape == (7, n)
        check_against_oracle(g, 7, lam.cpu().numpy(), vec.cpu().numpy().T.copy(), lam_full[:8], vec_full[:, :7])
        assert st["nconv"] == 7
    assert B.sc_workspace_bytes(n, int(rp[-1]), 7, m=80, block=4, guard=8) >= B.sc_workspace_bytes(n, int(rp[-1]), 7, m=80,
                                                                                                      block=4)
    with pytest.raises(B.ScError) as e:
        B.sc_laplacian_eigsh(drp, dc, dv, 7, 1e-10, guard=-1)
    assert e.value.code == B.SC_EDOMAIN
    with pytest.raises(B.ScError) as e:
        B.sc_laplacian_eigsh(drp, dc, dv, 7, 1e-10, guard=n)
    assert e.value.code == B.SC_EDOMAIN


def _asym_cases():
    g = wl.random_weighted_connected(300, 600, 2)
    rp, c, v, n = g
    cases = {}
    cases["symmetric"] = (rp, c, v, True)
    v2 = v.copy()
    v2[7] *= 1.0 + 1e-9                      # one direction of one edge changed in the ninth digit
    cases["one weight differs"] = (rp, c, v2, False)
    v3 = v.copy()
    rows = np.repeat(np.arange(n), np.diff(rp))
    e = 11
    back = np.flatnonzero((rows == c[e]) & (c == rows[e]))[0]
    v3[e] = v3[back] = -0.25                 # symmetric but negative
    cases["negative weight"] = (rp, c, v3, False)
    v4 = v.copy()
    v4[e] = v4[back] = np.inf
    cases["infinite weight"] = (rp, c, v4, False)
    # a directed edge: (0 -> 150) listed, (150 -> 0) not
    rows_l, cols_l, vals_l = list(rows), list(c), list(v)
    if not np.any((rows == 0) & (c == 150)):
        rows_l.append(0), cols_l.append(150), vals_l.append(0.5)
    g5 = wl.coo_to_csr(rows_l, cols_l, vals_l, n, sum_duplicates=False)
    cases["missing back edge"] = (g5[0], g5[1], g5[2], False)
    # symmetric, but columns in reverse order inside every row and one edge split into two entries per direction
    order = np.concatenate([np.arange(rp[i], rp[i + 1])[::-1] for i in range(n)])
    c6, v6 = c[order], v[order]
    rows6 = rows                      # row of every position is unchanged by a permutation inside rows
    e = 20
    i, j = rows6[e], c6[e]
    back = np.flatnonzero((rows6 == j) & (c6 == i))[0]
    rows_l = list(rows6) + [i, j]
    cols_l = list(c6) + [j, i]
    vals_l = list(v6) + [0.125, 0.125]
    # insert without sorting columns: build rowptr by counting, keep the listing order inside rows
    ordr = np.argsort(np.asarray(rows_l), kind="stable")
    rr = np.asarray(rows_l)[ordr]
    rp6 = np.zeros(n + 1, dtype=np.int64)
    rp6[1:] = np.cumsum(np.bincount(rr, minlength=n))
    cases["unsorted with a split edge"] = (rp6, np.asarray(cols_l, dtype=np.int32)[ordr], np.asarray(vals_l)[ordr], True)
    return cases, n


def test_symmetry_validation_flag(B):
    """SC_FLAG_VALIDATE_SYMMETRY: an asymmetric W, a negative or a non-finite weight give SC_ECSR and no output; a
    symmetric W passes whatever the order of its columns and however an edge is split into entries; without the flag
    nothing is checked (the precondition is the caller's)."""
    cases, n = _asym_cases()
    for name, (rp, c, v, ok) in cases.items():
        drp, dc, dv = B.csr_to_device(rp, c, v)
        if ok:
            lam, vec, code, _ = B.sc_laplacian_eigsh(drp, dc, dv, 3, 1e-9, flags=B.SC_FLAG_VALIDATE_SYMMETRY)
            assert code == B.SC_OK, name
            lam0, _ = dense.smallest_eigenpairs(rp, c, v, 3)
            assert np.max(np.abs(lam.cpu().numpy() - lam0)) <= 1e-8, name
        else:
            with pytest.raises(B.ScError) as e:
                B.sc_laplacian_eigsh(drp, dc, dv, 3, 1e-9, flags=B.SC_FLAG_VALIDATE_SYMMETRY)
            assert e.value.code == B.SC_ECSR, name
