"""GPU parity of every kernel-level step against the oracle's definitions, through the C ABI.

Sizes span several tiles (64-column MFMA tiles, 16/32-row tiles, 256-column workgroups, LDS chunks of
128/256 contraction indices) and ragged tails."""
import numpy as np
import pytest

from oracle import laplacian, blockops
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


def _graphs():
    cfg = wl.reduced(wl.CONFIGS[2], n=5003, components=7, k=7)
    g_knn, _, _ = wl.build_config_graph(cfg, device="cpu")
    return {"knn5003": g_knn, "ring1000": wl.ring(1000), "hub": _hub_graph(), "path2": wl.path(2)}


def _hub_graph():
    # one node connected to everybody (degree n-1 = 2999) on top of a ring: extreme row-length skew
    n = 3000
    i = np.arange(1, n)
    u = np.concatenate([np.zeros(n - 1, dtype=np.int64), i[:-1]])
    v = np.concatenate([i, i[1:]])
    w = np.random.default_rng(0).uniform(0.5, 2.0, size=u.size)
    return wl.symmetric_from_edges(u, v, w, n)


@pytest.fixture(scope="module")
def graphs():
    return _graphs()


def test_degree_scaling(B, graphs):
    for name, (rp, c, v, n) in graphs.items():
        drp, dc, dv = B.csr_to_device(rp, c, v)
        d, s = B.sc_degree_scaling(drp, dc, dv)
        d0 = laplacian.degrees(rp, c, v)
        assert np.allclose(d.cpu().numpy(), d0, rtol=1e-14, atol=0), name
        assert np.allclose(s.cpu().numpy(), 1.0 / np.sqrt(d0), rtol=1e-14, atol=0), name


def test_zero_degree_and_bad_csr_are_errors(B):
    rp = np.array([0, 1, 1, 2], dtype=np.int64)      # node 1 isolated
    c = np.array([2, 0], dtype=np.int32)
    v = np.array([1.0, 1.0])
    drp, dc, dv = B.csr_to_device(rp, c, v)
    with pytest.raises(B.ScError) as e:
        B.sc_degree_scaling(drp, dc, dv)
    assert e.value.code == B.SC_EZERODEG
    assert B.sc_validate_csr(drp, dc) == B.SC_OK
    bad_col = torch.tensor([2, 7], dtype=torch.int32, device="cuda")
    assert B.sc_validate_csr(drp, bad_col) == B.SC_ECSR
    bad_rp = torch.tensor([0, 2, 1, 2], dtype=torch.int64, device="cuda")
    assert B.sc_validate_csr(bad_rp, dc) == B.SC_ECSR
    neg = torch.tensor([1.0, -1.0], dtype=torch.float64, device="cuda")   # degree of node 2 = -1
    rp2 = torch.tensor([0, 1, 2], dtype=torch.int64, device="cuda")
    c2 = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    with pytest.raises(B.ScError) as e:
        B.sc_degree_scaling(rp2, c2, neg)
    assert e.value.code == B.SC_EZERODEG


@pytest.mark.parametrize("ncols", [1, 2, 4, 8, 16, 32])
def test_spmm_normalized(B, graphs, ncols):
    rng = np.random.default_rng(ncols)
    for name, (rp, c, v, n) in graphs.items():
        drp, dc, dv = B.csr_to_device(rp, c, v)
        _, s = B.sc_degree_scaling(drp, dc, dv)
        x = rng.standard_normal((n, ncols))
        # leading dimensions larger than ncols: the blocks live inside wider row-major buffers
        xb = torch.zeros((n, ncols + 3), dtype=torch.float64, device="cuda")
        xb[:, :ncols] = torch.from_numpy(x).cuda()
        yb = torch.full((n, ncols + 5), 7.0, dtype=torch.float64, device="cuda")
        B.sc_spmm_normalized(drp, dc, dv, s, xb[:, :ncols], yb[:, :ncols])
        y0 = laplacian.apply_s(rp, c, v, x)
        y = yb[:, :ncols].cpu().numpy()
        scale = np.abs(y0).max() + 1e-300
        assert np.max(np.abs(y - y0)) <= 1e-13 * scale, (name, ncols)
        assert torch.all(yb[:, ncols:] == 7.0)        # nothing written outside the block
        # caller-provided scratch: enqueue-only variant, result read after the stream is synchronised
        work = torch.empty((n, ncols), dtype=torch.float64, device="cuda")
        y2 = torch.zeros((n, ncols), dtype=torch.float64, device="cuda")
        B.sc_spmm_normalized(drp, dc, dv, s, xb[:, :ncols], y2, work)
        torch.cuda.synchronize()
        assert torch.equal(y2, yb[:, :ncols])


def _regular_with_hub(n, deg, seed):
    """Every node linked to its deg/2 successors on a ring (degree = deg everywhere), random weights, plus one hub
    joined to a quarter of the nodes: average degree close to deg, one row far longer than any register buffer."""
    rng = np.random.default_rng(seed)
    i = np.arange(n, dtype=np.int64)
    u = np.concatenate([i for _ in range(deg // 2)])
    v = np.concatenate([(i + t) % n for t in range(1, deg // 2 + 1)])
    far = np.arange(deg // 2 + 1, n - deg // 2 - 1, 4, dtype=np.int64)     # not already neighbours of node 0
    u = np.concatenate([u, np.zeros(far.size, dtype=np.int64)])
    v = np.concatenate([v, far])
    return wl.symmetric_from_edges(u, v, rng.uniform(0.5, 2.0, size=u.size), n)


@pytest.mark.parametrize("deg", [8, 18, 26, 36, 60, 100])
def test_single_vector_product_over_average_degrees(B, deg):
    """The single-vector product picks its tile height and register buffer from the average row length (six
    combinations, boundaries at about 14.8, 22.2, 29.6, 40.7 and 81.5 entries per row): one graph per combination,
    each with a hub row, with and without the scaling vector (the materialised operator), ragged last tile."""
    n = 4099
    rp, c, v, _ = _regular_with_hub(n, deg, deg)
    avg = rp[-1] / n
    assert deg <= avg < deg + 0.6
    drp, dc, dv = B.csr_to_device(rp, c, v)
    _, s = B.sc_degree_scaling(drp, dc, dv)
    x = np.random.default_rng(deg).standard_normal(n)
    y0 = laplacian.apply_s(rp, c, v, x)
    dx = torch.from_numpy(x).cuda()
    y = B.sc_spmm_normalized(drp, dc, dv, s, dx).cpu().numpy()
    assert np.max(np.abs(y - y0)) <= 1e-13 * np.abs(y0).max(), deg
    vs = B.sc_scale_operator(drp, dc, dv, s)
    y2 = B.sc_spmm_normalized(drp, dc, vs, None, dx)
    torch.cuda.synchronize()
    assert np.max(np.abs(y2.cpu().numpy() - y0)) <= 1e-13 * np.abs(y0).max(), deg


@pytest.mark.parametrize("deg", [4, 8, 26, 60])
def test_single_vector_product_chain(B, deg):
    """sc_spmv_normalized_chain: three products in a row, each taking the operand the previous one left (s o y), against
    the oracle's S applied three times; y of every link equals what sc_spmm_normalized gives for the same x."""
    n = 3001
    if deg == 4:
        rp, c, v, _ = wl.random_weighted_connected(n, 3000, 4)       # about 4 entries per row: the lanes-per-row kernel
    else:
        rp, c, v, _ = _regular_with_hub(n, deg, deg)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    _, s = B.sc_degree_scaling(drp, dc, dv)
    x = np.random.default_rng(deg).standard_normal(n)
    dx = torch.from_numpy(x).cuda()
    z = s * dx
    y = torch.empty_like(dx)
    z2 = torch.empty_like(dx)
    want = x
    for link in range(3):
        assert B.sc_spmv_normalized_chain(drp, dc, dv, s, int(rp[-1]), z, y, z2) == B.SC_OK
        torch.cuda.synchronize()
        want = laplacian.apply_s(rp, c, v, want)
        assert np.max(np.abs(y.cpu().numpy() - want)) <= 1e-13 * np.abs(want).max(), (deg, link)
        assert torch.equal(z2, s * y)
        z, z2 = z2, z
    with pytest.raises(B.ScError):
        B.sc_spmv_normalized_chain(drp, dc, dv, s, int(rp[-1]), z, y, z)


@pytest.mark.parametrize("ncols", [1, 2, 8, 16])
def test_scaled_operator_and_its_product(B, graphs, ncols):
    """Algorithm 2 step 3 as a step of its own: the scaled values are s_i w_ij s_j entry by entry and exactly symmetric,
    and the product with them (no scaling vector, operand gathered in place) is the oracle's S x."""
    rng = np.random.default_rng(100 + ncols)
    for name, (rp, c, v, n) in graphs.items():
        drp, dc, dv = B.csr_to_device(rp, c, v)
        _, s = B.sc_degree_scaling(drp, dc, dv)
        vs = B.sc_scale_operator(drp, dc, dv, s)
        s0 = laplacian.inv_sqrt_degrees(rp, c, v)
        rows = np.repeat(np.arange(n), np.diff(rp))
        want = s0[rows] * v * s0[c]
        got = vs.cpu().numpy()
        assert np.max(np.abs(got - want)) <= 4e-16 * np.max(np.abs(want)), name
        from scipy.sparse import csr_matrix
        a = csr_matrix((got, c, rp), shape=(n, n))
        assert abs(a - a.T).max() == 0.0, name                     # the same rounding for (i, j) and (j, i)
        x = rng.standard_normal((n, ncols))
        dx = torch.from_numpy(x).cuda()
        y = B.sc_spmm_normalized(drp, dc, vs, None, dx)
        torch.cuda.synchronize()
        y0 = laplacian.apply_s(rp, c, v, x)
        assert np.max(np.abs(y.cpu().numpy() - y0)) <= 1e-13 * (np.abs(y0).max() + 1e-300), (name, ncols)
        # an operand inside a wider buffer is packed first (no scaling), same answer
        xb = torch.zeros((n, ncols + 3), dtype=torch.float64, device="cuda")
        xb[:, :ncols] = dx
        y2 = B.sc_spmm_normalized(drp, dc, vs, None, xb[:, :ncols])
        torch.cuda.synchronize()
        assert torch.equal(y2, y), (name, ncols)


@pytest.mark.parametrize("shift", [0, 1, 2, 3])
def test_single_vector_product_on_offset_arrays(B, graphs, shift):
    """The single-vector product clamps its stream loads to the tile instead of predicating them: the same answer from
    (col, val) arrays that start 0..3 elements into a buffer (nothing before or after them is needed), on hub rows
    longer than the register buffer and on a graph of two rows."""
    rng = np.random.default_rng(shift)
    for name, (rp, c, v, n) in graphs.items():
        nnz = int(rp[-1])
        cbuf = torch.zeros(nnz + 8, dtype=torch.int32, device="cuda")
        vbuf = torch.zeros(nnz + 8, dtype=torch.float64, device="cuda")
        dc, dv = cbuf[shift:shift + nnz], vbuf[shift:shift + nnz]
        dc.copy_(torch.from_numpy(c))
        dv.copy_(torch.from_numpy(v))
        drp = torch.from_numpy(rp).cuda()
        _, s = B.sc_degree_scaling(drp, dc, dv)
        x = rng.standard_normal(n)
        y = B.sc_spmm_normalized(drp, dc, dv, s, torch.from_numpy(x).cuda()).cpu().numpy()
        y0 = laplacian.apply_s(rp, c, v, x)
        assert np.max(np.abs(y - y0)) <= 1e-13 * (np.abs(y0).max() + 1e-300), (name, shift)
        assert torch.all(cbuf[shift + nnz:] == 0) and torch.all(vbuf[:shift] == 0.0)


@pytest.mark.parametrize("n,j,b,pad", [(5000, 70, 16, 5), (4099, 130, 8, 5), (3001, 300, 32, 5), (2500, 17, 1, 5),
                                       (2000, 64, 4, 5), (777, 5, 2, 5), (70000, 200, 16, 5), (140000, 40, 32, 5),
                                       (300, 280, 8, 5),
                                       # rows of 32-byte multiples: the vector-load paths, as in the solver's basis
                                       (5000, 72, 16, 8), (3001, 300, 32, 4), (9000, 520, 32, 8)])
def test_cgs2(B, n, j, b, pad):
    rng = np.random.default_rng(n + j + b)
    q, _ = np.linalg.qr(rng.standard_normal((n, j)))
    w = rng.standard_normal((n, b)) + q @ rng.standard_normal((j, b)) * 3.0
    ld = j + b + pad
    basis = np.zeros((n, ld))
    basis[:, :j] = q
    basis[:, j:j + b] = w
    basis[:, j + b:] = 3.25
    dbasis = torch.from_numpy(basis).cuda()
    h, gram = B.sc_cgs2(dbasis, j, b, want_gram=True)
    w0, h0 = blockops.cgs2_block(q, w)
    g0 = w0.T @ w0
    assert np.max(np.abs(gram.cpu().numpy() - g0)) <= 1e-12 * np.abs(g0).max()
    out = dbasis.cpu().numpy()
    assert np.array_equal(out[:, :j], q) and np.all(out[:, j + b:] == 3.25)
    assert np.max(np.abs(h.cpu().numpy() - h0)) <= 1e-12 * max(1.0, np.abs(h0).max())
    assert np.max(np.abs(out[:, j:j + b] - w0)) <= 1e-12 * max(1.0, np.abs(w0).max())
    assert np.max(np.abs(q.T @ out[:, j:j + b])) <= 1e-13 * np.sqrt(n)


@pytest.mark.parametrize("n,j,b", [(5000, 0, 16), (4099, 7, 8), (3001, 40, 32), (2500, 3, 1), (999, 12, 4), (640, 2, 2)])
def test_block_qr(B, n, j, b):
    rng = np.random.default_rng(n + b)
    w = rng.standard_normal((n, b)) * np.logspace(0, -3, b)[None, :]   # columns of different scale
    ld = j + b + 2
    basis = rng.standard_normal((n, ld))
    basis[:, j:j + b] = w
    before = basis.copy()
    dbasis = torch.from_numpy(basis).cuda()
    r, g = B.sc_block_qr(dbasis, j, b)
    out = dbasis.cpu().numpy()
    q = out[:, j:j + b]
    r, g = r.cpu().numpy(), g.cpu().numpy()
    assert np.array_equal(out[:, :j], before[:, :j]) and np.array_equal(out[:, j + b:], before[:, j + b:])
    assert np.max(np.abs(q.T @ q - np.eye(b))) <= 1e-13
    assert np.allclose(np.tril(r, -1), 0.0)
    assert np.max(np.abs(q @ r - w)) <= 1e-12 * np.abs(w).max()
    assert np.max(np.abs(g - w.T @ w)) <= 1e-12 * np.abs(w.T @ w).max()


def test_block_qr_drops_dependent_and_zero_columns(B):
    n, b = 3000, 8
    rng = np.random.default_rng(5)
    w = rng.standard_normal((n, b))
    w[:, 3] = 2.0 * w[:, 0] - w[:, 2]        # dependent on earlier columns
    w[:, 6] = 0.0                             # zero column
    dbasis = torch.from_numpy(w.copy()).cuda()
    r, g = B.sc_block_qr(dbasis, 0, b)
    q = dbasis.cpu().numpy()
    r = r.cpu().numpy()
    keep = [0, 1, 2, 4, 5, 7]
    assert np.all(q[:, 3] == 0.0) and np.all(q[:, 6] == 0.0)
    assert np.all(r[3, :] == 0.0) and np.all(r[6, :] == 0.0)
    assert np.max(np.abs(q[:, keep].T @ q[:, keep] - np.eye(6))) <= 1e-13
    assert np.max(np.abs(q @ r - w)) <= 1e-11


@pytest.mark.parametrize("n,j0,ja,l,colmajor", [(5000, 0, 100, 40, False), (4099, 3, 77, 5, False),
                                                (3001, 8, 300, 130, True), (1000, 1, 16, 1, True),
                                                (2048, 4, 520, 64, False)])
def test_rotate(B, n, j0, ja, l, colmajor):
    rng = np.random.default_rng(n + ja)
    basis = rng.standard_normal((n, j0 + ja + 3))
    y = rng.standard_normal((ja, l))
    dbasis = torch.from_numpy(basis).cuda()
    out = B.sc_rotate(dbasis, j0, ja, torch.from_numpy(y).cuda(), out_colmajor=colmajor).cpu().numpy()
    ref = blockops.rotate(basis[:, j0:j0 + ja], y)
    if colmajor:
        out = out.T
    assert np.max(np.abs(out - ref)) <= 1e-12 * np.abs(ref).max()


def test_reorder_csr_is_a_permutation_similarity(B):
    from oracle import components
    parts = [wl.ring(30), wl.path(41), wl.random_weighted_connected(200, 500, 3), wl.hypercube(5)]
    g = wl.disjoint_union(*parts)
    g = wl.relabel(g, np.random.default_rng(3).permutation(g[3]))
    rp, c, v, n = g
    drp, dc, dv = B.csr_to_device(rp, c, v)
    rp2, c2, v2, oon, ncomp = B.sc_reorder_csr(drp, dc, dv)
    assert ncomp == len(parts) == components.component_labels(rp, c, v)[0]
    oon = oon.cpu().numpy().astype(np.int64)
    assert np.array_equal(np.sort(oon), np.arange(n))
    from scipy.sparse import csr_matrix
    a = csr_matrix((v, c, rp), shape=(n, n)).toarray()
    a2 = csr_matrix((v2.cpu().numpy(), c2.cpu().numpy(), rp2.cpu().numpy()), shape=(n, n)).toarray()
    assert np.array_equal(a2, a[np.ix_(oon, oon)])                 # A'[p, q] = A[old(p), old(q)], bit for bit
    _, label = components.component_labels(rp, c, v)
    lab_new = label[oon]
    assert np.all(np.diff(np.flatnonzero(np.diff(lab_new) != 0)) > 0) and len(set(lab_new)) == ncomp
    # every component is one contiguous run
    assert np.count_nonzero(np.diff(lab_new) != 0) == ncomp - 1


@pytest.mark.parametrize("ncols", [1, 4, 8, 16, 32])
def test_chebyshev_filter(B, ncols):
    """The start-block filter as a step of its own against the oracle's three-term recurrence: a graph that spans
    several row tiles with a ragged tail, hub rows longer than one batch, both code paths (narrow blocks on W and s,
    wide blocks on the scaled copy with the recurrence fused into the product)."""
    from oracle import blockops
    rng = np.random.default_rng(40 + ncols)
    # complete(70) gives rows of 69 entries (three batches of a 32-lane group); complete(300) and the star's centre
    # give rows of 299 and 500 entries, beyond the 128 above which the wide products hand a row to a whole workgroup
    star = wl.symmetric_from_edges(np.zeros(500, dtype=np.int64), np.arange(1, 501), np.linspace(0.5, 1.5, 500), 501)
    g = wl.disjoint_union(wl.random_weighted_connected(700, 9000, 5), wl.ring(257), wl.complete(70),
                          wl.random_weighted_connected(333, 700, 6), wl.complete(300), star)
    g = wl.relabel(g, rng.permutation(g[3]))
    rp, c, v, n = g
    assert np.sum(np.diff(rp) > 128) == 301
    x = rng.standard_normal((n, ncols))
    a, d = 0.4, 12
    want = blockops.chebyshev_filter(rp, c, v, x, a, d)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    got = B.sc_chebyshev_filter(drp, dc, dv, torch.from_numpy(x).cuda(), a, d).cpu().numpy()
    scale = np.max(np.abs(want))
    assert scale > 1e3                                   # the polynomial did amplify the top of the spectrum
    assert np.max(np.abs(got - want)) <= 1e-11 * scale   # d products and a three-term recurrence in fp64
    # degree 1 is the plain affine image of S
    got1 = B.sc_chebyshev_filter(drp, dc, dv, torch.from_numpy(x).cuda(), a, 1).cpu().numpy()
    assert np.max(np.abs(got1 - blockops.chebyshev_filter(rp, c, v, x, a, 1))) <= 1e-13 * max(1.0, np.max(np.abs(x)))


def _block_diagonal_graph():
    """Contiguous diagonal blocks of every kind the LDS-resident filter distinguishes: two rows; fewer rows than a wave
    has lane groups; rows of 1, 2, 27 (average), 33, 69 and 500 entries (one chunk, several chunks, a hub spread over
    16 or 32 lane groups); more chunks than lane groups (second chunk slot); 300 to 501 rows (too many for 32 columns
    at once: two 16-column items)."""
    star = wl.symmetric_from_edges(np.zeros(500, dtype=np.int64), np.arange(1, 501), np.linspace(0.5, 1.5, 500), 501)
    return wl.disjoint_union(wl.path(2), wl.random_weighted_connected(300, 4000, 5), wl.ring(257), wl.complete(70),
                             wl.ring(7), wl.random_weighted_connected(333, 700, 6), star, wl.complete(34),
                             wl.random_weighted_connected(450, 2500, 7), wl.path(31))


@pytest.mark.parametrize("ncols", [16, 32])
@pytest.mark.parametrize("degree", [1, 2, 12])
def test_chebyshev_filter_resident_in_lds(B, ncols, degree, monkeypatch):
    """The one-launch form of the start-block filter (a workgroup keeps the iterates of a diagonal block in LDS and the
    block's entries in registers through all steps) against the oracle's recurrence, element by element, on a
    block-diagonal graph as given; it must be the path taken (event counter), be bitwise repeatable, and agree with the
    product-per-step path to rounding."""
    from oracle import blockops
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")       # small graph: the cost model would pick the other path
    g = _block_diagonal_graph()
    rp, c, v, n = g
    assert np.diff(rp).max() == 500 and np.sum(np.diff(rp) > 32) > 100
    rng = np.random.default_rng(7 * ncols + degree)
    x = rng.standard_normal((n, ncols))
    a = 0.4
    want = blockops.chebyshev_filter(rp, c, v, x, a, degree)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    dx = torch.from_numpy(x).cuda()
    before = B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS)
    got = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before + 1
    scale = max(1.0, np.max(np.abs(want)))
    assert np.max(np.abs(got.cpu().numpy() - want)) <= 1e-11 * scale
    again = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert torch.equal(got, again)
    monkeypatch.delenv("SCEIG_FORCE_RESIDENT")
    monkeypatch.setenv("SCEIG_NO_RESIDENT", "1")
    other = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before + 2
    assert np.max(np.abs(other.cpu().numpy() - got.cpu().numpy())) <= 1e-11 * scale
    # the input block inside a wider buffer
    monkeypatch.delenv("SCEIG_NO_RESIDENT")
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")
    xb = torch.zeros((n, ncols + 3), dtype=torch.float64, device="cuda")
    xb[:, :ncols] = dx
    got2 = B.sc_chebyshev_filter(drp, dc, dv, xb[:, :ncols], a, degree)
    assert torch.equal(got2, got)


@pytest.mark.parametrize("ncols", [16, 32])
@pytest.mark.parametrize("degree", [2, 12])
def test_chebyshev_filter_resident_sliced_form(B, ncols, degree, monkeypatch):
    """Diagonal blocks of 700 to 1,150 rows: too many rows (or entries) for the form that keeps the entries in
    registers, so they go as 8-column items that stream their entries from a sliced copy (slices of 64 rows, the last
    one of a block shorter; rows of 2 to 50 entries, so slices with padding); small blocks in the same matrix keep the
    register form.  Against the oracle's recurrence element by element, bitwise repeatable, and it must be the
    one-launch path."""
    from oracle import blockops
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")
    rp, c, v, n = wl.disjoint_union(wl.random_weighted_connected(700, 9000, 1), wl.path(2), wl.ring(1150),
                                    wl.random_weighted_connected(1000, 16000, 2), wl.complete(40), wl.path(65))
    rng = np.random.default_rng(11 * ncols + degree)
    x = rng.standard_normal((n, ncols))
    a = 0.35
    want = blockops.chebyshev_filter(rp, c, v, x, a, degree)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    dx = torch.from_numpy(x).cuda()
    before = B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS)
    got = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before + 1
    scale = max(1.0, np.max(np.abs(want)))
    assert np.max(np.abs(got.cpu().numpy() - want)) <= 1e-11 * scale
    assert torch.equal(got, B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree))
    # without the sliced form these blocks do not fit, and the product-per-step path gives the same to rounding
    monkeypatch.setenv("SCEIG_NO_SLICED", "1")
    other = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before + 2
    assert np.max(np.abs(other.cpu().numpy() - want)) <= 1e-11 * scale


@pytest.mark.parametrize("degree", [1, 2, 3, 8])
def test_chebyshev_filter_resident_with_trailing_large_blocks(B, degree, monkeypatch):
    """Blocks too large for any item (1,300 and 1,400 rows) at the END of the matrix: the items of the other blocks go
    in one launch, the trailing rows step by step through the product kernel restricted to them (long rows among them
    included), and both land in the same result; degrees 1, 2, 3 cover the three buffers the last step can end in."""
    from oracle import blockops
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")
    star = wl.symmetric_from_edges(np.zeros(500, dtype=np.int64), np.arange(1, 501), np.linspace(0.5, 1.5, 500), 501)
    rp, c, v, n = wl.disjoint_union(wl.random_weighted_connected(700, 9000, 1), wl.ring(300), star,
                                    wl.random_weighted_connected(1300, 5000, 3),
                                    wl.disjoint_union(wl.random_weighted_connected(1400, 30000, 4)))
    big_star = wl.symmetric_from_edges(np.zeros(1500, dtype=np.int64), np.arange(1, 1501), np.ones(1500), 1501)
    rp, c, v, n = wl.disjoint_union((rp, c, v, n), big_star)      # a trailing block with a row of 1,500 entries
    rng = np.random.default_rng(degree)
    x = rng.standard_normal((n, 16))
    a = 0.3
    want = blockops.chebyshev_filter(rp, c, v, x, a, degree)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    dx = torch.from_numpy(x).cuda()
    before = B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS)
    got = B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree)
    assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before + 1
    assert np.max(np.abs(got.cpu().numpy() - want)) <= 1e-11 * max(1.0, np.max(np.abs(want)))
    assert torch.equal(got, B.sc_chebyshev_filter(drp, dc, dv, dx, a, degree))


def test_chebyshev_filter_resident_declines_what_does_not_fit(B, monkeypatch):
    """A block with more rows than LDS holds even as 8-column items (1,300 rows) that is NOT at the end of the matrix,
    or a block width without a resident form (8 columns): the product-per-step way, even when the resident form is
    asked for; the answer is the oracle's either way."""
    from oracle import blockops
    monkeypatch.setenv("SCEIG_FORCE_RESIDENT", "1")
    rng = np.random.default_rng(3)
    cases = [(wl.disjoint_union(wl.random_weighted_connected(1300, 5000, 1), wl.ring(40)), 16),
             (wl.disjoint_union(wl.ring(40), wl.ring(50)), 8)]
    for (rp, c, v, n), ncols in cases:
        x = rng.standard_normal((n, ncols))
        drp, dc, dv = B.csr_to_device(rp, c, v)
        before = B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS)
        got = B.sc_chebyshev_filter(drp, dc, dv, torch.from_numpy(x).cuda(), 0.3, 5).cpu().numpy()
        assert B.sc_counter(B.SC_COUNTER_RESIDENT_FILTERS) == before
        want = blockops.chebyshev_filter(rp, c, v, x, 0.3, 5)
        assert np.max(np.abs(got - want)) <= 1e-11 * max(1.0, np.max(np.abs(want)))


def test_chebyshev_filter_rejects_bad_arguments(B):
    rp, c, v, n = wl.ring(20)
    drp, dc, dv = B.csr_to_device(rp, c, v)
    x = torch.zeros((n, 8), dtype=torch.float64, device="cuda")
    for a, d in ((1.0, 3), (-1.0, 3), (0.3, 0)):
        with pytest.raises(B.ScError):
            B.sc_chebyshev_filter(drp, dc, dv, x, a, d)


def test_fp64_matrix_rate_probe(B):
    """The measurement aid runs in both forms of the instruction, reports rates that the published fp64 matrix peak
    bounds, and refuses bad arguments."""
    import ctypes
    for shape in (16, 4):
        rate = B.sc_probe_fp64_matrix_rate(512, 500, shape)
        assert 1.0 < rate <= 78.6 * 1.05, (shape, rate)
    out = ctypes.c_double(0.0)
    assert B.lib().sc_probe_fp64_matrix_rate(16, 0, 10, ctypes.byref(out), 0) == B.SC_EDOMAIN
    assert B.lib().sc_probe_fp64_matrix_rate(16, 8, 0, ctypes.byref(out), 0) == B.SC_EDOMAIN
    assert B.lib().sc_probe_fp64_matrix_rate(8, 8, 8, ctypes.byref(out), 0) == B.SC_EDOMAIN
    assert B.lib().sc_probe_fp64_matrix_rate(16, 8, 8, None, 0) == B.SC_EINVAL
