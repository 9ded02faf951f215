"""Shared parity checks between the HIP solver's output and the oracle's (host side, numpy fp64)."""
import numpy as np

from oracle import compare

TOL_EVAL = 1e-8      # |lambda_gpu - lambda_oracle|
TOL_RESID = 1e-6     # ||L v - lambda v||_2 per pair, recomputed here
TOL_ANGLE = 1e-5     # rad, largest principal angle per separated cluster


def check_against_oracle(graph, k, lam_gpu, vec_gpu, lam_oracle_ext, vec_oracle, cluster_basis=None):
    """lam_oracle_ext: at least k+1 ascending oracle eigenvalues (or exactly k if the (k+1)-th is unknown);
    vec_oracle: oracle eigenvectors for the first k.  cluster_basis: optional orthonormal basis of a space that
    must contain the GPU vectors when k cuts a cluster (e.g. the closed-form null space)."""
    rp, c, v, n = graph
    lam_gpu = np.asarray(lam_gpu)
    vec_gpu = np.asarray(vec_gpu)
    assert lam_gpu.shape == (k,) and vec_gpu.shape == (n, k)
    assert np.all(np.isfinite(lam_gpu)) and np.all(np.isfinite(vec_gpu))
    assert np.all(np.diff(lam_gpu) >= -1e-12), "eigenvalues must ascend"
    dlam = np.max(np.abs(lam_gpu - lam_oracle_ext[:k]))
    assert dlam <= TOL_EVAL, f"eigenvalue mismatch {dlam}"
    assert lam_gpu.min() > -1e-10 and lam_gpu.max() < 2.0 + 1e-10
    res = compare.residual_norms(rp, c, v, lam_gpu, vec_gpu)
    assert res.max() <= TOL_RESID, f"residual {res.max()}"
    assert compare.orthonormality_defect(vec_gpu) <= 1e-9
    out = {"max_dlam": float(dlam), "max_resid": float(res.max()), "max_angle": 0.0, "max_contain": 0.0}
    if len(lam_oracle_ext) > k:
        res_o = compare.residual_norms(rp, c, v, lam_oracle_ext[:k], vec_oracle[:, :k])
        runs = compare.separated_clusters(np.asarray(lam_oracle_ext), k, float(res.max() + res_o.max()))
        for a, b in runs:
            ang = compare.principal_angles(vec_gpu[:, a:b], vec_oracle[:, a:b])
            out["max_angle"] = max(out["max_angle"], float(ang.max()))
            assert ang.max() <= TOL_ANGLE, f"cluster [{a},{b}) angle {ang.max()}"
        out["clusters"] = runs
    if cluster_basis is not None:
        defect = compare.containment_defect(vec_gpu, cluster_basis)
        out["max_contain"] = float(defect.max())
        assert defect.max() <= TOL_ANGLE, f"containment {defect.max()}"
    return out
