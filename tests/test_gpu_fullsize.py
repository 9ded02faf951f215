"""Full-size runs of the three large workloads (configs 3, 4, 5) against the exact component oracle.

These take minutes each (most of it building the synthetic kNN graph), so they only run when
SCEIG_FULLSIZE names them, e.g.  SCEIG_FULLSIZE=3,5 python -m pytest tests/test_gpu_fullsize.py -m gpu -s.
The benchmark workload (config 2) at full size is in tests/test_gpu_eigsh.py and always runs.

Reference at this size (a plain Lanczos oracle would need hours): the graphs are unions of connected components,
so the wanted eigenvalues are exactly 0 (multiplicity = number of components >= k, checked by union-find) and the
eigenspace is spanned by D^1/2 1_C / sqrt(vol C).  Checks: |lambda| <= 1e-8, residuals recomputed on the host
<= 1e-6, containment of every GPU vector in the closed-form null space <= 1e-5, orthonormality on a sample."""
import os
import sys
import time

import numpy as np
import pytest

from oracle import components, laplacian
from paper_1802_04450_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

WANTED = {int(t) for t in os.environ.get("SCEIG_FULLSIZE", "").replace(" ", "").split(",") if t}


def say(*a):
    print(*a, file=sys.stderr, flush=True)


@pytest.mark.parametrize("cid", [3, 4, 5])
def test_fullsize_workload(cid):
    if cid not in WANTED:
        pytest.skip("set SCEIG_FULLSIZE=%d to run this multi-minute case" % cid)
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_1802_04450_amd import binding as B
    from scipy.sparse import csr_matrix
    cfg = wl.CONFIGS[cid]
    t0 = time.time()
    g, label, sigma = wl.build_config_graph(cfg, device="cuda")
    rp, c, v, n = g
    say(f"[cfg{cid}] graph {wl.describe(g)} sigma={sigma:.4g} built in {time.time() - t0:.0f}s")
    t0 = time.time()
    ncomp, comp = components.component_labels(rp, c, v)
    say(f"[cfg{cid}] components={ncomp} ({time.time() - t0:.0f}s)")
    block = int(os.environ.get("SCEIG_BLOCK", "0"))
    # Config 4 (global sigma on anisotropic blobs) has a ladder of eigenvalues 1e-11 ... 1e-6 directly above the
    # exact zeros; resolving it by Lanczos alone needs tens of thousands of steps per phase, so this run locks the
    # closed-form null vectors of the connected components first (the library's optional pre-pass) and lets the
    # Lanczos check phase confirm that nothing above them is missing.
    default_flags = B.SC_FLAG_COMPONENT_NULLSPACE if cid == 4 else 0
    flags = int(os.environ.get("SCEIG_FLAGS", str(default_flags)))
    drp, dc, dv = B.csr_to_device(rp, c, v)
    t0 = time.time()
    evals, evecs, code, stats = B.sc_laplacian_eigsh(drp, dc, dv, cfg.k, cfg.tol, m=cfg.m, block=block, flags=flags,
                                                     timing_mask=63)
    torch.cuda.synchronize()
    say(f"[cfg{cid}] solve {time.time() - t0:.2f}s code={code} stats={stats}")
    assert code == B.SC_OK
    lam = evals.cpu().numpy()
    say(f"[cfg{cid}] lambda min={lam.min():.3e} max={lam.max():.3e}")
    kzero = min(cfg.k, ncomp)
    assert np.all(np.diff(lam) >= -1e-12)
    assert np.max(np.abs(lam[:kzero])) <= 1e-8
    # host-side checks on column chunks (the full n x k block is up to 8 GB)
    d = laplacian.degrees(rp, c, v)
    s = 1.0 / np.sqrt(d)
    w = csr_matrix((v, c, rp), shape=(n, n))
    vol = np.bincount(comp, weights=d, minlength=ncomp)
    nullcoef = np.sqrt(d / vol[comp])                    # the single nonzero of each row of the null basis
    nbasis = csr_matrix((nullcoef, (np.arange(n), comp)), shape=(n, ncomp))
    rng = np.random.default_rng(0)
    sample = np.sort(rng.choice(cfg.k, size=min(cfg.k, 48), replace=False))
    xs = evecs[torch.from_numpy(sample).cuda()].cpu().numpy().T          # n x |sample|
    worst_res = worst_def = 0.0
    chunk = 100
    gram_rows = []
    for c0 in range(0, cfg.k, chunk):
        x = evecs[c0:c0 + chunk].cpu().numpy().T
        sx = s[:, None] * (w @ (s[:, None] * x))
        res = np.linalg.norm(x - sx - x * lam[None, c0:c0 + chunk], axis=0)
        worst_res = max(worst_res, float(res.max()))
        if c0 + x.shape[1] <= kzero:
            inside = nbasis @ (nbasis.T @ x)
            worst_def = max(worst_def, float(np.linalg.norm(x - inside, axis=0).max()))
        gram_rows.append(xs.T @ x)
    gram = np.concatenate(gram_rows, axis=1)             # |sample| x k
    eye = np.zeros_like(gram)
    eye[np.arange(sample.size), sample] = 1.0
    ortho = float(np.max(np.abs(gram - eye)))
    say(f"[cfg{cid}] max residual={worst_res:.3e} containment defect={worst_def:.3e} orthonormality={ortho:.3e}")
    assert worst_res <= 1e-6
    assert worst_def <= 1e-5
    assert ortho <= 1e-9
