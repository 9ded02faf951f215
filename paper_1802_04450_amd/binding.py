"""ctypes binding of libsceig.so (include/sceig.h): argument marshalling only.

Device buffers are torch CUDA(HIP) tensors; their ``data_ptr()`` and the current torch stream are
handed to the library.  Nothing here computes: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsceig.so")

SC_OK, SC_NOT_CONVERGED = 0, 1
SC_EINVAL, SC_EDOMAIN, SC_ECSR, SC_EZERODEG, SC_ENOMEM, SC_EHIP, SC_EINTERNAL = -1, -2, -3, -4, -5, -6, -7
SC_FLAG_NO_VERIFY = 1
SC_FLAG_NO_REORDER = 2
SC_FLAG_COMPONENT_NULLSPACE = 4
SC_FLAG_NO_START_FILTER = 8
SC_FLAG_FINAL_RR = 16
SC_FLAG_RANDOM_WALK_VECTORS = 32
SC_FLAG_ROW_NORMALIZE = 64
SC_FLAG_VALIDATE_SYMMETRY = 128
FAMILIES = ["spmm", "project", "update", "rotate", "qr", "other"]

EXPORTS = ["sc_laplacian_eigsh", "sc_degree_scaling", "sc_spmm_normalized", "sc_validate_csr", "sc_reorder_csr", "sc_cgs2",
           "sc_block_qr", "sc_rotate", "sc_sym_eig", "sc_sym_eig_top", "sc_strerror", "sc_version", "sc_release_cache",
           "sc_chebyshev_filter", "sc_kmeanspp", "sc_kmeans_lloyd", "sc_kmeans", "sc_edge_similarity", "sc_knn_search", "sc_knn_union_pairs",
           "sc_coo_to_csr", "sc_workspace_bytes", "sc_scale_operator", "sc_laplacian_eigsh_ws",
           "sc_block_qr_noalloc", "sc_counter",
           "sc_spmv_normalized_chain", "sc_probe_fp64_matrix_rate"]


class ScOptions(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("block", ctypes.c_int32), ("check_every", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("seed", ctypes.c_uint64), ("timing_mask", ctypes.c_uint32),
                ("guard", ctypes.c_int32), ("v0", ctypes.c_void_p)]


class ScStats(ctypes.Structure):
    _fields_ = [("nconv", ctypes.c_int32), ("phases", ctypes.c_int32), ("restarts", ctypes.c_int32),
                ("block", ctypes.c_int32), ("m", ctypes.c_int32), ("host_eigs", ctypes.c_int32),
                ("components", ctypes.c_int32), ("filter_steps", ctypes.c_int32),
                ("block_steps", ctypes.c_int64), ("spmv_cols", ctypes.c_int64), ("t_total", ctypes.c_double),
                ("t_host_eig", ctypes.c_double), ("t_setup", ctypes.c_double), ("max_residual_est", ctypes.c_double),
                ("fam_time_s", ctypes.c_double * 6), ("fam_bytes", ctypes.c_double * 6),
                ("fam_flops", ctypes.c_double * 6), ("fam_launches", ctypes.c_int64 * 6)]

    def as_dict(self) -> dict:
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            out[name] = list(v) if name.startswith("fam_") else v
        return out


class ScKMeansStats(ctypes.Structure):
    _fields_ = [("iterations", ctypes.c_int32), ("converged", ctypes.c_int32), ("last_changes", ctypes.c_int32),
                ("timing", ctypes.c_int32), ("objective", ctypes.c_double), ("t_total", ctypes.c_double),
                ("t_seed", ctypes.c_double), ("t_distance", ctypes.c_double), ("distance_launches", ctypes.c_int64),
                ("distance_bytes", ctypes.c_double), ("distance_flops", ctypes.c_double)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class ScError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sceig error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (build it first with ``python -m paper_1802_04450_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_1802_04450_amd.build`")
        # torch ships its own HIP runtime (same soname as the one this library links against).  Loading torch
        # first makes the dynamic loader bind the library to that copy, so that torch's device pointers and
        # streams are valid inside the library; two runtimes in one process do not see each other's memory.
        import torch  # noqa: F401
        _lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        _lib.sc_laplacian_eigsh.argtypes = [vp, vp, vp, i64, i32, dbl, i32, vp, vp, vp, ctypes.POINTER(ScOptions),
                                            ctypes.POINTER(ScStats)]
        _lib.sc_laplacian_eigsh_ws.argtypes = [vp, vp, vp, i64, i32, dbl, i32, vp, vp, vp, ctypes.POINTER(ScOptions),
                                               ctypes.POINTER(ScStats), vp, ctypes.c_size_t]
        _lib.sc_workspace_bytes.argtypes = [i64, i64, i32, ctypes.POINTER(ScOptions), ctypes.POINTER(ctypes.c_size_t)]
        _lib.sc_degree_scaling.argtypes = [vp, vp, vp, i64, vp, vp, vp]
        _lib.sc_scale_operator.argtypes = [vp, vp, vp, vp, i64, vp, vp]
        _lib.sc_spmm_normalized.argtypes = [vp, vp, vp, vp, i64, vp, i64, vp, i64, i32, vp, vp]
        _lib.sc_validate_csr.argtypes = [vp, vp, i64, vp]
        _lib.sc_spmv_normalized_chain.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, vp, vp]
        _lib.sc_reorder_csr.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_int32), vp]
        _lib.sc_cgs2.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        _lib.sc_block_qr.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        _lib.sc_block_qr_noalloc.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        _lib.sc_rotate.argtypes = [vp, i64, i64, i32, i32, vp, i32, vp, i64, i32, vp]
        _lib.sc_chebyshev_filter.argtypes = [vp, vp, vp, i64, vp, i64, i32, dbl, i32, vp, i64, vp]
        u64 = ctypes.c_uint64
        _lib.sc_kmeanspp.argtypes = [vp, i64, i32, i64, i32, i32, u64, vp, vp, vp]
        _lib.sc_kmeans_lloyd.argtypes = [vp, i64, i32, i64, i32, i32, vp, i32, vp, ctypes.POINTER(ScKMeansStats), vp]
        _lib.sc_kmeans.argtypes = [vp, i64, i32, i64, i32, i32, u64, i32, vp, vp, ctypes.POINTER(ScKMeansStats), vp]
        _lib.sc_edge_similarity.argtypes = [vp, i64, i64, i32, vp, vp, i64, i32, dbl, vp, vp]
        _lib.sc_coo_to_csr.argtypes = [vp, vp, vp, i64, i64, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_int64), vp]
        _lib.sc_knn_search.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        _lib.sc_knn_union_pairs.argtypes = [vp, vp, i64, i32, dbl, vp, vp, vp, ctypes.POINTER(ctypes.c_int64), vp]
        _lib.sc_sym_eig.argtypes = [vp, i32, vp, vp]
        _lib.sc_sym_eig_top.argtypes = [vp, i32, i32, vp, vp]
        for name in EXPORTS:
            getattr(_lib, name).restype = ctypes.c_int
        _lib.sc_strerror.restype = ctypes.c_char_p
        _lib.sc_strerror.argtypes = [ctypes.c_int]
        _lib.sc_version.argtypes = []
        _lib.sc_release_cache.argtypes = []
        _lib.sc_counter.argtypes = [ctypes.c_int32]
        _lib.sc_probe_fp64_matrix_rate.argtypes = [i32, i32, i32, ctypes.POINTER(ctypes.c_double), vp]
        _lib.sc_counter.restype = ctypes.c_int64
    return _lib


SC_COUNTER_RESIDENT_FILTERS = 0


def sc_counter(which: int) -> int:
    """Process-wide event counter of the library (host only)."""
    return int(lib().sc_counter(which))


def sc_probe_fp64_matrix_rate(workgroups: int = 2048, iterations: int = 4000, shape: int = 16) -> float:
    """TFLOP/s of a launch that issues only fp64 matrix-core instructions (the practical ceiling of that rate);
    shape 16 = the 16x16x4 form, 4 = the 4x4x4 form."""
    out = ctypes.c_double(0.0)
    _check(lib().sc_probe_fp64_matrix_rate(shape, workgroups, iterations, ctypes.byref(out), _stream()))
    return float(out.value)


def sc_release_cache() -> int:
    """Give the device and pinned blocks the library keeps between calls back to the HIP runtime."""
    return int(lib().sc_release_cache())


def strerror(code: int) -> str:
    return lib().sc_strerror(code).decode()


def _check(code: int, soft_ok: bool = True) -> int:
    if code < 0 or (code > 0 and not soft_ok):
        raise ScError(code, strerror(code))
    return code


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _dev(t, dtype):
    import torch
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype, t.is_contiguous())
    return t


def csr_to_device(rowptr: np.ndarray, col: np.ndarray, val: np.ndarray, device="cuda:0"):
    """Host CSR arrays -> (rowptr int64, col int32, val fp64) device tensors."""
    import torch
    return (torch.from_numpy(np.ascontiguousarray(rowptr, dtype=np.int64)).to(device),
            torch.from_numpy(np.ascontiguousarray(col, dtype=np.int32)).to(device),
            torch.from_numpy(np.ascontiguousarray(val, dtype=np.float64)).to(device))


# ----------------------------------------------------------------------------------------------
def sc_laplacian_eigsh(rowptr, col, val, k: int, tol: float, maxiter: int = 100000, m: int = 0, block: int = 0,
                       check_every: int = 0, flags: int = 0, seed: int = 0, timing_mask: int = 0, guard: int = 0,
                       v0=None, workspace=None, out=None):
    """Returns (evals[k] device, evecs (k, n) device - row t is eigenvector t, i.e. the library's
    column-major n x k output -, status code, stats dict).  workspace: a device tensor that the solve works inside
    (sc_laplacian_eigsh_ws); out: (evals, evecs) tensors to write into instead of new ones."""
    import torch
    n = rowptr.numel() - 1
    _dev(rowptr, torch.int64), _dev(col, torch.int32), _dev(val, torch.float64)
    if out is None:
        evals = torch.empty(max(k, 0), dtype=torch.float64, device=rowptr.device)
        evecs = torch.empty((max(k, 0), n), dtype=torch.float64, device=rowptr.device)
    else:
        evals, evecs = out
        _dev(evals, torch.float64), _dev(evecs, torch.float64)
        assert evals.numel() >= k and evecs.numel() >= k * n
    if v0 is not None:
        _dev(v0, torch.float64)
        assert v0.numel() == n
    opt = ScOptions(m=m, block=block, check_every=check_every, flags=flags, seed=seed, timing_mask=timing_mask,
                    guard=guard, v0=_ptr(v0))
    stats = ScStats()
    with torch.cuda.device(rowptr.device):
        if workspace is None:
            code = lib().sc_laplacian_eigsh(_ptr(rowptr), _ptr(col), _ptr(val), n, k, tol, maxiter, _ptr(evals),
                                            _ptr(evecs), _stream(), ctypes.byref(opt), ctypes.byref(stats))
        else:
            assert workspace.is_cuda and workspace.is_contiguous()
            code = lib().sc_laplacian_eigsh_ws(_ptr(rowptr), _ptr(col), _ptr(val), n, k, tol, maxiter, _ptr(evals),
                                               _ptr(evecs), _stream(), ctypes.byref(opt), ctypes.byref(stats),
                                               _ptr(workspace), workspace.numel() * workspace.element_size())
    _check(code)
    return evals, evecs, code, stats.as_dict()


def sc_workspace_bytes(n: int, nnz: int, k: int, m: int = 0, block: int = 0, flags: int = 0, guard: int = 0) -> int:
    """Device bytes a solve of this size allocates for itself (host-only query)."""
    opt = ScOptions(m=m, block=block, flags=flags, guard=guard)
    out = ctypes.c_size_t(0)
    _check(lib().sc_workspace_bytes(n, nnz, k, ctypes.byref(opt), ctypes.byref(out)), soft_ok=False)
    return int(out.value)


def sc_degree_scaling(rowptr, col, val, want_degrees: bool = True):
    import torch
    n = rowptr.numel() - 1
    d = torch.empty(n, dtype=torch.float64, device=rowptr.device) if want_degrees else None
    s = torch.empty(n, dtype=torch.float64, device=rowptr.device)
    with torch.cuda.device(rowptr.device):
        code = lib().sc_degree_scaling(_ptr(rowptr), _ptr(col), _ptr(val), n, _ptr(d), _ptr(s), _stream())
    _check(code)
    return d, s


def sc_spmv_normalized_chain(rowptr, col, val, s, nnz: int, z_in, y, z_out):
    """One product of a chain: y = s o (W z_in), z_out = s o y, with z_in = s o x from the previous product.  Only
    enqueues on the current stream; y and z_out are written in place.  Returns the status code."""
    import torch
    n = rowptr.numel() - 1
    for t in (s, z_in, y, z_out):
        _dev(t, torch.float64)
        assert t.numel() == n
    with torch.cuda.device(rowptr.device):
        code = lib().sc_spmv_normalized_chain(_ptr(rowptr), _ptr(col), _ptr(val), _ptr(s), n, nnz, _ptr(z_in), _ptr(y),
                                              _ptr(z_out), _stream())
    return _check(code)


def sc_scale_operator(rowptr, col, val, s):
    """Algorithm 2 step 3, symmetric form: a new value array S_ij = s_i W_ij s_j."""
    import torch
    n = rowptr.numel() - 1
    out = torch.empty_like(val)
    with torch.cuda.device(rowptr.device):
        code = lib().sc_scale_operator(_ptr(rowptr), _ptr(col), _ptr(val), _ptr(s), n, _ptr(out), _stream())
    _check(code)
    return out


def sc_validate_csr(rowptr, col) -> int:
    import torch
    n = rowptr.numel() - 1
    with torch.cuda.device(rowptr.device):
        return lib().sc_validate_csr(_ptr(rowptr), _ptr(col), n, _stream())


def sc_reorder_csr(rowptr, col, val):
    """Component-contiguous renumbering.  Returns (rowptr', col', val', old_of_new int32[n], ncomp)."""
    import torch
    n = rowptr.numel() - 1
    rp2, c2, v2 = torch.empty_like(rowptr), torch.empty_like(col), torch.empty_like(val)
    oon = torch.empty(n, dtype=torch.int32, device=rowptr.device)
    ncomp = ctypes.c_int32(0)
    with torch.cuda.device(rowptr.device):
        code = lib().sc_reorder_csr(_ptr(rowptr), _ptr(col), _ptr(val), n, _ptr(rp2), _ptr(c2), _ptr(v2), _ptr(oon),
                                    ctypes.byref(ncomp), _stream())
    _check(code)
    return rp2, c2, v2, oon, int(ncomp.value)


def sc_spmm_normalized(rowptr, col, val, s, x, y=None, work=None):
    """x: (n, ncols) row-major device tensor (a 1-D tensor is one column).  Returns y of the same shape.
    s=None: `val` holds the scaled operator from sc_scale_operator and y = S x is one launch.
    With `work` given (or s=None and a packed x) the call only enqueues on the current stream (synchronise before
    reading y on the host)."""
    import torch
    n = rowptr.numel() - 1
    x2 = x.reshape(n, -1)
    ncols = x2.shape[1]
    if y is None:
        y = torch.empty_like(x2)
    y2 = y.reshape(n, -1)
    with torch.cuda.device(rowptr.device):
        code = lib().sc_spmm_normalized(_ptr(rowptr), _ptr(col), _ptr(val), _ptr(s), n, _ptr(x2), x2.stride(0),
                                        _ptr(y2), y2.stride(0), ncols, _ptr(work), _stream())
    _check(code)
    return y.reshape(x.shape)


def sc_cgs2(basis, j: int, b: int, want_h: bool = True, want_gram: bool = False):
    """basis: (n, ld) row-major device tensor, columns j..j+b-1 updated in place.  Returns H (j, b) or None;
    with want_gram also the Gram matrix (b, b) of the updated block."""
    import torch
    n, ld = basis.shape
    h = torch.zeros((j, b), dtype=torch.float64, device=basis.device) if want_h else None
    g = torch.zeros((b, b), dtype=torch.float64, device=basis.device) if want_gram else None
    with torch.cuda.device(basis.device):
        code = lib().sc_cgs2(_ptr(basis), n, basis.stride(0), j, b, _ptr(h), _ptr(g), _stream())
    _check(code)
    return (h, g) if want_gram else h


def sc_block_qr(basis, j: int, b: int):
    """In-place Cholesky-QR (twice) of columns j..j+b-1.  Returns (R (b, b), G (b, b))."""
    import torch
    n, ld = basis.shape
    r = torch.zeros((b, b), dtype=torch.float64, device=basis.device)
    g = torch.zeros((b, b), dtype=torch.float64, device=basis.device)
    with torch.cuda.device(basis.device):
        code = lib().sc_block_qr(_ptr(basis), n, basis.stride(0), j, b, _ptr(r), _ptr(g), _stream())
    _check(code)
    return r, g


def sc_block_qr_noalloc(basis, j: int, b: int, r, g):
    """sc_block_qr on the library's fixed device scratch: the call allocates nothing, so the outputs r and g ((b, b)
    device tensors) are the caller's.  Returns the status code."""
    n, ld = basis.shape
    with __import__("torch").cuda.device(basis.device):
        code = lib().sc_block_qr_noalloc(_ptr(basis), n, basis.stride(0), j, b, _ptr(r), _ptr(g), _stream())
    return _check(code)


def sc_rotate(basis, j0: int, ja: int, y, out_colmajor: bool = False):
    """basis[:, j0:j0+ja] @ y  with y (ja, l) row-major.  Returns (n, l) row-major, or (l, n) if out_colmajor."""
    import torch
    n, ld = basis.shape
    l = y.shape[1]
    yc = y.contiguous()
    if out_colmajor:
        out = torch.empty((l, n), dtype=torch.float64, device=basis.device)
        ldo = n
    else:
        out = torch.empty((n, l), dtype=torch.float64, device=basis.device)
        ldo = l
    with torch.cuda.device(basis.device):
        code = lib().sc_rotate(_ptr(basis), n, basis.stride(0), j0, ja, _ptr(yc), l, _ptr(out), ldo,
                               1 if out_colmajor else 0, _stream())
    _check(code)
    return out


def sc_chebyshev_filter(rowptr, col, val, x, a: float, degree: int):
    """T_degree(g(S)) x for a row-major (n, ncols) block x, g mapping [-1, a] to [-1, 1].  Returns a new (n, ncols) tensor."""
    import torch
    n = rowptr.numel() - 1
    ncols = x.shape[1]
    y = torch.empty((n, ncols), dtype=torch.float64, device=x.device)
    with torch.cuda.device(x.device):
        code = lib().sc_chebyshev_filter(_ptr(rowptr), _ptr(col), _ptr(val), n, _ptr(x), x.stride(0), ncols,
                                         float(a), int(degree), _ptr(y), ncols, _stream())
    _check(code)
    return y


def _points_layout(points, colmajor: bool):
    """(n, d, ld) of a 2-d device tensor holding the points: shape (n, d) row-major, or shape (d, n) with
    colmajor=True (row t = coordinate t of every point, the layout sc_laplacian_eigsh returns)."""
    import torch
    _dev(points, torch.float64)
    if colmajor:
        d, n = points.shape
    else:
        n, d = points.shape
    return n, d, points.stride(0)


def sc_kmeanspp(points, k: int, seed: int, colmajor: bool = False):
    """Algorithm 5.  Returns (chosen int32[k] device, centres (k, d) device)."""
    import torch
    n, d, ld = _points_layout(points, colmajor)
    chosen = torch.empty(max(k, 0), dtype=torch.int32, device=points.device)
    cen = torch.empty((max(k, 0), d), dtype=torch.float64, device=points.device)
    with torch.cuda.device(points.device):
        code = lib().sc_kmeanspp(_ptr(points), ld, 1 if colmajor else 0, n, d, k, seed, _ptr(chosen), _ptr(cen),
                                 _stream())
    _check(code)
    return chosen, cen


def sc_kmeans_lloyd(points, centroids, max_iter: int = 100, colmajor: bool = False, timing: bool = False):
    """Algorithm 4 step 3 from `centroids` ((k, d) device, not modified).  Returns (labels int32[n], centres (k, d),
    status code, stats dict)."""
    import torch
    n, d, ld = _points_layout(points, colmajor)
    cen = _dev(centroids, torch.float64).clone()
    k = cen.shape[0]
    labels = torch.empty(n, dtype=torch.int32, device=points.device)
    stats = ScKMeansStats(timing=1 if timing else 0)
    with torch.cuda.device(points.device):
        code = lib().sc_kmeans_lloyd(_ptr(points), ld, 1 if colmajor else 0, n, d, k, _ptr(cen), max_iter,
                                     _ptr(labels), ctypes.byref(stats), _stream())
    _check(code)
    return labels, cen, code, stats.as_dict()


def sc_kmeans(points, k: int, seed: int, max_iter: int = 100, colmajor: bool = False, timing: bool = False):
    """Algorithm 4.  Returns (labels int32[n], centres (k, d), status code, stats dict)."""
    import torch
    n, d, ld = _points_layout(points, colmajor)
    labels = torch.empty(n, dtype=torch.int32, device=points.device)
    cen = torch.empty((max(k, 0), d), dtype=torch.float64, device=points.device)
    stats = ScKMeansStats(timing=1 if timing else 0)
    with torch.cuda.device(points.device):
        code = lib().sc_kmeans(_ptr(points), ld, 1 if colmajor else 0, n, d, k, seed, max_iter, _ptr(labels),
                               _ptr(cen), ctypes.byref(stats), _stream())
    _check(code)
    return labels, cen, code, stats.as_dict()


SC_SIM_CROSS_CORRELATION, SC_SIM_COSINE, SC_SIM_EXP_DECAY = 0, 1, 2


def sc_edge_similarity(x, edge_u, edge_v, measure: int, sigma: float = 1.0):
    """Algorithm 1: similarity of the listed pairs of rows of x ((n, d) device).  Returns val fp64[nedges] device."""
    import torch
    _dev(x, torch.float64), _dev(edge_u, torch.int32), _dev(edge_v, torch.int32)
    n, d = x.shape
    ne = edge_u.numel()
    val = torch.empty(ne, dtype=torch.float64, device=x.device)
    with torch.cuda.device(x.device):
        code = lib().sc_edge_similarity(_ptr(x), x.stride(0), n, d, _ptr(edge_u), _ptr(edge_v), ne, measure,
                                        float(sigma), _ptr(val), _stream())
    _check(code)
    return val


def sc_coo_to_csr(row, col, val, n: int, symmetrize: bool):
    """Algorithm 2 step 4.  Returns (rowptr int64[n+1], col int32[nnz], val fp64[nnz]) device, sorted by (row, col)."""
    import torch
    _dev(row, torch.int32), _dev(col, torch.int32), _dev(val, torch.float64)
    nnz_in = row.numel()
    total = nnz_in * (2 if symmetrize else 1)
    rp = torch.empty(n + 1, dtype=torch.int64, device=row.device)
    co = torch.empty(max(total, 1), dtype=torch.int32, device=row.device)
    vo = torch.empty(max(total, 1), dtype=torch.float64, device=row.device)
    nnz = ctypes.c_int64(0)
    with torch.cuda.device(row.device):
        code = lib().sc_coo_to_csr(_ptr(row), _ptr(col), _ptr(val), nnz_in, n, 1 if symmetrize else 0, _ptr(rp), _ptr(co),
                                   _ptr(vo), ctypes.byref(nnz), _stream())
    _check(code)
    return rp, co[:nnz.value], vo[:nnz.value]


def sc_knn_search(x, k_nn: int):
    """Section III-A's k nearest neighbours of every row of x ((n, d) device).  Returns (idx int32 (n, k_nn),
    dist fp64 (n, k_nn)) device, nearest first."""
    import torch
    _dev(x, torch.float64)
    n, d = x.shape
    idx = torch.empty((n, k_nn), dtype=torch.int32, device=x.device)
    dist = torch.empty((n, k_nn), dtype=torch.float64, device=x.device)
    with torch.cuda.device(x.device):
        code = lib().sc_knn_search(_ptr(x), x.stride(0), n, d, k_nn, _ptr(idx), _ptr(dist), _stream())
    _check(code)
    return idx, dist


def sc_knn_union_pairs(idx, dist, sigma: float = 0.0):
    """The undirected edges of the kNN graph, each once.  Returns (edge_u, edge_v int32, val fp64) device."""
    import torch
    _dev(idx, torch.int32), _dev(dist, torch.float64)
    n, k_nn = idx.shape
    assert idx.is_contiguous() and dist.is_contiguous() and dist.shape == idx.shape
    eu = torch.empty(max(n * k_nn, 1), dtype=torch.int32, device=idx.device)
    ev = torch.empty(max(n * k_nn, 1), dtype=torch.int32, device=idx.device)
    val = torch.empty(max(n * k_nn, 1), dtype=torch.float64, device=idx.device)
    npairs = ctypes.c_int64(0)
    with torch.cuda.device(idx.device):
        code = lib().sc_knn_union_pairs(_ptr(idx), _ptr(dist), n, k_nn, float(sigma), _ptr(eu), _ptr(ev), _ptr(val),
                                        ctypes.byref(npairs), _stream())
    _check(code)
    m = npairs.value
    return eu[:m], ev[:m], val[:m]


def sc_sym_eig(a: np.ndarray, vectors: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Host projected eigenproblem: eigenvalues ascending and eigenvectors (columns) of a symmetric matrix."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    n = a.shape[0]
    w = np.empty(n)
    z = np.empty((n, n)) if vectors else None
    code = lib().sc_sym_eig(a.ctypes.data, n, w.ctypes.data, z.ctypes.data if vectors else 0)
    _check(code, soft_ok=False)
    return w, z


def sc_sym_eig_top(a: np.ndarray, count: int) -> Tuple[np.ndarray, np.ndarray]:
    """All eigenvalues (ascending) and the eigenvectors of the `count` largest (column t <-> w[n-1-t])."""
    a = np.ascontiguousarray(a, dtype=np.float64)
    n = a.shape[0]
    w = np.empty(n)
    z = np.empty((n, max(count, 1)))
    code = lib().sc_sym_eig_top(a.ctypes.data, n, count, w.ctypes.data, z.ctypes.data)
    _check(code, soft_ok=False)
    return w, z[:, :count]
