"""Full-size runs of the three large workloads (configs 3, 4, 5) against the exact component oracle.

Collected by default (the benchmark workload, config 2, at full size is in tests/test_gpu_eigsh.py).  Most of each
case's time is building the synthetic kNN graph; SCEIG_FULLSIZE=3,5 restricts the run to the named configs.

Reference at this size (a plain Lanczos oracle would need hours): the graphs are unions of connected components,
so the wanted eigenvalues are exactly 0 (multiplicity = number of components >= k, checked by union-find) and the
eigenspace is spanned by D^1/2 1_C / sqrt(vol C).  Checks: |lambda| <= 1e-8, residuals recomputed on the host
<= 1e-6, containment of every GPU vector in the closed-form null space <= 1e-5, orthonormality on a sample.

Config 4 (4,000,000 nodes) gets three runs, each named for what it is:
  * plain path, Gaussian weights, bounded number of restart cycles: the honest status of Algorithm 3's loop on a graph
    whose spectrum has a ladder of eigenvalues 1e-11 ... 1e-6 right above the 200 zeros (no Lanczos method separates
    them at tol = 1e-7 within minutes); the run must execute sparse products and reorthogonalizations at k = 200,
    m = 400 and report what it reached;
  * plain path, unit weights on the same edges (a clean gap after the zeros): full parity against the component oracle;
  * SC_FLAG_COMPONENT_NULLSPACE: the closed-form null vectors of the components, locked by the optional pre-pass after
    their residuals have been formed with block products.  This run takes no Lanczos step; it is a check of the
    pre-pass, not of the hot path."""
import os
import sys
import time

import numpy as np
import pytest

from oracle import components, laplacian
from paper_1802_04450_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

ONLY = {int(t) for t in os.environ.get("SCEIG_FULLSIZE", "").replace(" ", "").split(",") if t}


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def wanted(cid):
    if ONLY and cid not in ONLY:
        pytest.skip("SCEIG_FULLSIZE names other configs")
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")


class HostChecks:
    """Host-side quantities of one graph that every check of it needs (oracle degrees, closed-form null basis)."""

    def __init__(self, graph, tag):
        from scipy.sparse import csr_matrix
        rp, c, v, n = graph
        self.n, self.tag = n, tag
        t0 = time.time()
        self.ncomp, comp = components.component_labels(rp, c, v)
        say(f"[{tag}] components={self.ncomp} ({time.time() - t0:.0f}s)")
        d = laplacian.degrees(rp, c, v)
        self.s = 1.0 / np.sqrt(d)
        self.w = csr_matrix((v, c, rp), shape=(n, n))
        vol = np.bincount(comp, weights=d, minlength=self.ncomp)
        coef = np.sqrt(d / vol[comp])                     # the single nonzero of each row of the null basis
        self.nbasis = csr_matrix((coef, (np.arange(n), comp)), shape=(n, self.ncomp))

    def measure(self, lam, evecs, k, kzero):
        """Residuals ||L x - lambda x||, containment defect in the null space (first kzero vectors) and orthonormality
        on a sample of columns, in column chunks (the full n x k block is up to 8 GB).  evecs: device (k, n)."""
        rng = np.random.default_rng(0)
        sample = np.sort(rng.choice(k, size=min(k, 48), replace=False))
        xs = evecs[torch.from_numpy(sample).cuda()].cpu().numpy().T
        res_all = np.empty(k)
        self.rayleigh_gap = 0.0                            # max |lambda_t - x_t^T L x_t|
        worst_def = 0.0
        gram_rows = []
        for c0 in range(0, k, 100):
            x = evecs[c0:c0 + 100].cpu().numpy().T
            sx = self.s[:, None] * (self.w @ (self.s[:, None] * x))
            res_all[c0:c0 + x.shape[1]] = np.linalg.norm(x - sx - x * lam[None, c0:c0 + x.shape[1]], axis=0)
            rq = np.sum(x * (x - sx), axis=0)
            self.rayleigh_gap = max(self.rayleigh_gap, float(np.max(np.abs(rq - lam[c0:c0 + x.shape[1]]))))
            if c0 + x.shape[1] <= kzero:
                inside = self.nbasis @ (self.nbasis.T @ x)
                worst_def = max(worst_def, float(np.linalg.norm(x - inside, axis=0).max()))
            gram_rows.append(xs.T @ x)
        gram = np.concatenate(gram_rows, axis=1)
        eye = np.zeros_like(gram)
        eye[np.arange(sample.size), sample] = 1.0
        return res_all, worst_def, float(np.max(np.abs(gram - eye)))


def solve_and_check(B, cfg, graph, host, tag, flags=0, block=0, maxiter=3000, must_converge=True):
    rp, c, v, n = graph
    drp, dc, dv = B.csr_to_device(rp, c, v)
    t0 = time.time()
    evals, evecs, code, stats = B.sc_laplacian_eigsh(drp, dc, dv, cfg.k, cfg.tol, maxiter=maxiter, m=cfg.m, block=block,
                                                     flags=flags, timing_mask=63)
    torch.cuda.synchronize()
    say(f"[{tag}] solve {time.time() - t0:.2f}s code={code} stats={stats}")
    lam = evals.cpu().numpy()
    say(f"[{tag}] lambda min={lam.min():.3e} max={lam.max():.3e}")
    kzero = min(cfg.k, host.ncomp)
    res, worst_def, ortho = host.measure(lam, evecs, cfg.k, kzero if must_converge else 0)
    say(f"[{tag}] max residual={res.max():.3e} containment defect={worst_def:.3e} orthonormality={ortho:.3e} "
        f"Rayleigh-quotient gap={host.rayleigh_gap:.3e}")
    assert np.all(np.isfinite(lam)) and np.all(np.diff(lam) >= -1e-12)
    assert ortho <= 1e-9
    assert host.rayleigh_gap <= 1e-9
    if must_converge:
        assert code == B.SC_OK
        assert np.max(np.abs(lam[:kzero])) <= 1e-8
        assert res.max() <= 1e-6
        assert worst_def <= 1e-5
    del drp, dc, dv, evecs
    B.sc_release_cache()
    torch.cuda.empty_cache()
    return lam, res, code, stats


@pytest.mark.parametrize("cid", [3, 5])
def test_fullsize_workload(cid):
    """Configs 3 (k = 500 cuts the null space of ~1000 components) and 5 (k = 2000, m = 4000, block 32) through the plain
    path: products, CGS2, block QR, restarts, locking, output."""
    wanted(cid)
    from paper_1802_04450_amd import binding as B
    cfg = wl.CONFIGS[cid]
    t0 = time.time()
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    say(f"[cfg{cid}] graph {wl.describe(g)} sigma={sigma:.4g} built in {time.time() - t0:.0f}s")
    host = HostChecks(g, f"cfg{cid}")
    assert host.ncomp >= cfg.k
    block = int(os.environ.get("SCEIG_BLOCK", "0"))
    lam, res, code, stats = solve_and_check(B, cfg, g, host, f"cfg{cid}", block=block)
    assert stats["block_steps"] > 0 and stats["spmv_cols"] > 0
    if cid == 5 and block == 0:
        assert stats["block"] == 32


@pytest.fixture(scope="module")
def cfg4():
    wanted(4)
    cfg = wl.CONFIGS[4]
    t0 = time.time()
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    say(f"[cfg4] graph {wl.describe(g)} sigma={sigma:.4g} built in {time.time() - t0:.0f}s")
    return cfg, g, HostChecks(g, "cfg4")


def test_config4_plain_path_bounded(cfg4):
    """Gaussian weights, default options, at most 120 restart cycles.  SC_NOT_CONVERGED is an accepted, stated outcome:
    what is required is that the hot path ran at full size (products and reorthogonalizations counted), that the
    output is finite, ascending and orthonormal, that every pair the solver counts as converged has a recomputed
    residual within the parity bar, and that every returned value is the Rayleigh quotient of its vector."""
    from paper_1802_04450_amd import binding as B
    cfg, g, host = cfg4
    lam, res, code, stats = solve_and_check(B, cfg, g, host, "cfg4 plain", maxiter=120, must_converge=False)
    assert code in (B.SC_OK, B.SC_NOT_CONVERGED)
    assert stats["block_steps"] >= 100 and stats["spmv_cols"] >= 100 * stats["block"]
    assert stats["m"] == 400 and stats["block"] == 16
    assert lam.min() > -1e-10 and lam.max() < 2.0
    nconv = int(stats["nconv"])
    say(f"[cfg4 plain] status={B.strerror(code)} nconv={nconv} of {cfg.k}; recomputed residuals: "
        f"min {res.min():.2e} median {np.median(res):.2e} max {res.max():.2e}; "
        f"{int((res <= 1e-6).sum())} of {cfg.k} within 1e-6")
    assert int((res <= 1e-6).sum()) >= nconv
    if code == B.SC_OK:
        assert nconv == cfg.k and res.max() <= 1e-6


def test_config4_unit_weights_plain_path(cfg4):
    """Secondary run, labelled as such: config 4's edges with unit weights.  Same 200 components, but the ladder of
    near-zero eigenvalues that the global Gaussian bandwidth creates is gone (the next eigenvalue is about 0.009), so
    the plain path converges; full parity against the component oracle (closed-form null space).  tol = 1e-8 instead
    of the workload's 1e-7: the containment bar of 1e-5 rad needs residual / gap <= 1e-5, and 1e-7 / 0.009 is just
    above it (measured 1.06e-5 at tol = 1e-7)."""
    import dataclasses
    from paper_1802_04450_amd import binding as B
    cfg, g, _ = cfg4
    cfg = dataclasses.replace(cfg, tol=1e-8)
    rp, c, v, n = g
    gu = (rp, c, np.ones_like(v), n)
    host = HostChecks(gu, "cfg4 unit")
    assert host.ncomp >= cfg.k
    lam, res, code, stats = solve_and_check(B, cfg, gu, host, "cfg4 unit")
    assert stats["block_steps"] > 0 and stats["spmv_cols"] > 0 and stats["phases"] > 0


def test_config4_component_nullspace_prepass(cfg4):
    """SC_FLAG_COMPONENT_NULLSPACE on the Gaussian-weight graph: the pre-pass locks D^1/2 1_C / sqrt(vol C) for the 200
    components (each after its residual ||S v - v|| met tol) and the solver returns them.  No Lanczos step runs
    (block_steps = 0): this is the shortcut, not the hot path; the vectors are verified here by recomputed residuals and
    containment."""
    from paper_1802_04450_amd import binding as B
    cfg, g, host = cfg4
    assert host.ncomp >= cfg.k
    lam, res, code, stats = solve_and_check(B, cfg, g, host, "cfg4 prepass", flags=B.SC_FLAG_COMPONENT_NULLSPACE)
    assert stats["components"] == host.ncomp and stats["block_steps"] == 0 and stats["spmv_cols"] == cfg.k
