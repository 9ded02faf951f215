#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A "step" is one complete eigensolve (sc_laplacian_eigsh: setup, block Lanczos, final Ritz vectors) of the
benchmark workload with the CSR graph already resident in HBM.  Prints ONE JSON line.

The headline workload is the largest one, config 5 (n = 500,000, k = 2,000, m = 4,000: a 16 GB basis, the
reorthogonalization-dominated case), through the plain path.  The default run adds, as extra keys of the same line,
the eigensolve seconds of configs 1, 2 and 3 (`per_config`), the single-vector product on the 4,000,000-node graph of
config 4 (`spmv_large`: the only size at which the product is bandwidth-bound), a complete run of the CPU oracle on
config 2 (`cpu_baseline_cfg2`) and an extrapolated oracle time for the headline workload (`cpu_baseline`).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg2|...] [--no-extras] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP64_MFMA_PEAK_TFLOPS = 78.6
KERNEL_OF_FAMILY = ["spmm_cols_kernel / cheb_resident_kernel (S X with fused D^-1/2 scaling; filter steps)",
                    "project_kernel (CGS2 block projection H = Q^T W, fp64 MFMA)",
                    "row_gemm_kernel mode 0 / update_gram_kernel (CGS2 block update W -= Q H, fp64 MFMA)",
                    "row_gemm_kernel mode 1/2 (restart rotation V Y, fp64 MFMA)",
                    "block QR (Gram + Cholesky + scaling)", "reduce_partials_kernel"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# kernel-name prefix of each timed family in the committed rocprofv3 traffic summary (sorted by total time, so the
# first match is the family's dominant kernel)
TRAFFIC_PREFIX = ["spmm_", "project_kernel", ("row_gemm_kernel", "update_gram_kernel"), "row_gemm_kernel",
                  ("apply_gram_kernel", "apply_rinv_kernel", "chol_reg_kernel"), "reduce_partials_kernel"]


def profiled_traffic(workload: str, family: int):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by the plain-copy calibration) of the family's dominant
    kernel, from the rocprofv3 counter summary committed for this workload.  The summary records the hash of the kernel
    sources it was measured on; when that is not the tree's hash (or there is no summary) the figure is None: a
    counter reading of other code is not a measurement of this run."""
    from paper_1802_04450_amd.build import source_hash
    path = os.path.join(ROOT, "profiles", f"{workload}_eigensolve_traffic.txt")
    if not os.path.exists(path):
        return None, None, "no counter summary for this workload", None
    recorded, rows = None, []
    for line in open(path):
        if line.startswith("# csrc_sha256:"):
            recorded = line.split(":", 1)[1].strip()
        elif line.strip() and not line.startswith("#"):
            rows.append(line.split())
    if recorded != source_hash():
        return None, None, "counter summary was measured on other kernel sources", None
    for row in rows:
        name, fetch, write, avg = row[0], row[1], row[2], row[3]
        if name.startswith(TRAFFIC_PREFIX[family]):
            extra = {"avg_launch_us_profiled": float(avg), "mfma_f64_flops_per_launch": float(row[4]) if len(row) > 4 else 0.0}
            return float(fetch) + float(write), name, f"profiles/{workload}_eigensolve_traffic.txt", extra
    return None, None, "kernel not in the counter summary", None


def build_workload(name: str):
    from paper_1802_04450_amd import workloads as wl
    t0 = time.time()
    if name in wl.SECOND_WORKLOADS:  # connected graphs of the shape of the paper's own datasets (not the headline)
        import types
        graph, spec = wl.build_second_workload(name)
        cfg = types.SimpleNamespace(name=name, n=spec["n"], k=spec["k"], m=spec.get("m", 0), tol=spec["tol"])
        log(f"[bench] built {name}: {wl.describe(graph)} in {time.time() - t0:.1f}s")
        return cfg, graph
    cid = int(name.replace("cfg", ""))
    cfg = wl.CONFIGS[cid]
    graph, label, sigma = wl.build_config_graph(cfg, device="cuda")
    log(f"[bench] built {cfg.name}: {wl.describe(graph)} sigma={sigma:.4g} in {time.time() - t0:.1f}s")
    return cfg, graph


def host_threads() -> int:
    try:
        import threadpoolctl
        return int(max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline_full(cfg, graph):
    """The oracle as it stands, run to the end on this workload (same graph, tolerance and basis budget)."""
    from oracle import lanczos
    rp, c, v, n = graph
    t0 = time.time()
    lam, vec, info = lanczos.lanczos_smallest(rp, c, v, k=cfg.k, tol=cfg.tol, m=cfg.m or None, seed=0, return_info=True)
    dt = time.time() - t0
    return {"value": dt, "unit": "s", "cores": host_threads(), "kind": "oracle",
            "sample": f"one complete oracle solve of {cfg.name} (k={cfg.k}, m={cfg.m}, tol={cfg.tol}): {info['spmv']} SpMV, "
                      f"{info['phases']} phases, converged={info['converged']}, largest |lambda| {float(np.max(np.abs(lam))):.1e}"}


def cpu_baseline_extrapolated(cfg, graph):
    """For the workloads whose complete oracle run takes hours: the oracle's own pieces timed at the real size -
    its Lanczos for the first few pairs (steps per pair), its sparse product, and its twice-applied Gram-Schmidt
    against k/2 stored vectors (the average number over a solve that locks one pair per phase) - and
    steps x seconds-per-step from them.  Labelled as an extrapolation."""
    from oracle import lanczos, laplacian
    rp, c, v, n = graph
    ks = 3
    t0 = time.time()
    lam, vec, info = lanczos.lanczos_smallest(rp, c, v, k=ks, tol=cfg.tol, m=cfg.m or None, seed=0, return_info=True)
    dt_few = time.time() - t0
    steps_per_pair = info["spmv"] / max(1, info["locked"])
    op = laplacian.NormalizedOperator(rp, c, v)
    rng = np.random.default_rng(0)
    x = rng.standard_normal(n)
    t0 = time.time()
    for _ in range(3):
        op(x)
    t_spmv = (time.time() - t0) / 3
    j = max(1, min(cfg.k // 2, int(3.0e9 / (8 * n))))       # stored vectors of the timed reorthogonalization (<= 3 GB)
    basis = rng.standard_normal((n, j))
    t0 = time.time()
    lanczos._cgs2(x.copy(), [basis])
    t_cgs2_j = time.time() - t0
    t_cgs2 = t_cgs2_j * (cfg.k / 2) / j                     # linear in the number of stored vectors
    steps = steps_per_pair * cfg.k
    return {"value": steps * (t_spmv + t_cgs2), "unit": "s", "cores": host_threads(), "kind": "oracle-extrapolated",
            "sample": f"oracle Lanczos for the first {info['locked']} pairs: {info['spmv']} steps in {dt_few:.1f}s "
                      f"({steps_per_pair:.1f} steps per pair); oracle product {t_spmv * 1e3:.1f} ms; oracle CGS2 against "
                      f"{j} vectors {t_cgs2_j * 1e3:.0f} ms, scaled to the average {cfg.k // 2}; value = {steps:.0f} steps x "
                      f"{(t_spmv + t_cgs2) * 1e3:.0f} ms (no complete oracle run at this size: it would take hours)"}


def measure_spmv(B, torch, drp, dc, dv, n, nnz):
    """Single-vector y = S x: algorithmic bytes / time, on the node numbering the solver itself works in (its setup
    pass makes every connected component contiguous and orders each by neighbourhood min-hash; that pass is part of
    every timed eigensolve) and, for context, on the numbering the caller handed over.  Products are enqueued back to
    back."""
    def time_spmv(rp_d, c_d, v_d):
        _, s = B.sc_degree_scaling(rp_d, c_d, v_d, want_degrees=False)
        x = torch.randn(n, dtype=torch.float64, device="cuda")
        y = torch.empty_like(x)
        work = torch.empty_like(x)
        for _ in range(5):
            B.sc_spmm_normalized(rp_d, c_d, v_d, s, x, y, work)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 50
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            B.sc_spmm_normalized(rp_d, c_d, v_d, s, x, y, work)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def time_spmv_scaled(rp_d, c_d, v_d):
        """The same product on the materialised operator S_ij = s_i W_ij s_j (Algorithm 2's ScaleElements): one launch, no
        scaling vector and no scaling pass."""
        _, s = B.sc_degree_scaling(rp_d, c_d, v_d, want_degrees=False)
        vs = B.sc_scale_operator(rp_d, c_d, v_d, s)
        x = torch.randn(n, dtype=torch.float64, device="cuda")
        y = torch.empty_like(x)
        for _ in range(5):
            B.sc_spmm_normalized(rp_d, c_d, vs, None, x, y)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 50
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            B.sc_spmm_normalized(rp_d, c_d, vs, None, x, y)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def time_spmv_chain(rp_d, c_d, v_d):
        """The product as it occurs in a chain (sc_spmv_normalized_chain): the operand arrives scaled by the previous
        product, which also leaves the next operand; one launch per product, both scalings fused, no scaling pass."""
        _, s = B.sc_degree_scaling(rp_d, c_d, v_d, want_degrees=False)
        x = torch.randn(n, dtype=torch.float64, device="cuda")
        za, zb = s * x, torch.empty_like(x)
        y = torch.empty_like(x)
        for _ in range(5):
            B.sc_spmv_normalized_chain(rp_d, c_d, v_d, s, nnz, za, y, zb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 50
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps // 2):       # the two operand buffers alternate; the values stay bounded (|S| = 1)
            B.sc_spmv_normalized_chain(rp_d, c_d, v_d, s, nnz, za, y, zb)
            B.sc_spmv_normalized_chain(rp_d, c_d, v_d, s, nnz, zb, y, za)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / (2 * (reps // 2))

    rp2, c2, v2, _, ncomp = B.sc_reorder_csr(drp, dc, dv)
    spmv_s = time_spmv(rp2, c2, v2)
    spmv_s_chain = time_spmv_chain(rp2, c2, v2)
    spmv_s_scaled = time_spmv_scaled(rp2, c2, v2)
    spmv_s_given = time_spmv(drp, dc, dv)
    spmv_bytes = 12 * nnz + 8 * (n + 1) + 8 * n + 8 * n + 8 * n
    scaled_bytes = 12 * nnz + 8 * (n + 1) + 8 * n + 8 * n
    chain_bytes = spmv_bytes + 8 * n          # the next operand is written as well
    spmv_gbs = spmv_bytes / spmv_s / 1e9
    return {"gbps_algorithmic": spmv_gbs, "seconds": spmv_s, "bytes": spmv_bytes,
            "frac_of_hbm_peak": spmv_gbs / HBM_PEAK_GBS,
            "chain": {"gbps_algorithmic": chain_bytes / spmv_s_chain / 1e9, "seconds": spmv_s_chain,
                      "bytes": chain_bytes, "frac_of_hbm_peak": chain_bytes / spmv_s_chain / 1e9 / HBM_PEAK_GBS,
                      "note": "y = s o (W (s o x)) inside a chain of products (sc_spmv_normalized_chain): one launch, the "
                              "operand arrives scaled by the previous product, which also writes the next operand"},
            "scaled_operator": {"gbps_algorithmic": scaled_bytes / spmv_s_scaled / 1e9, "seconds": spmv_s_scaled,
                                "bytes": scaled_bytes,
                                "frac_of_hbm_peak": scaled_bytes / spmv_s_scaled / 1e9 / HBM_PEAK_GBS,
                                "note": "y = S x on the materialised operator (sc_scale_operator), one launch"},
            "gbps_algorithmic_caller_numbering": spmv_bytes / spmv_s_given / 1e9, "components": int(ncomp),
            "note": "single-vector y = S x (prescale pass + product kernel), 50 back-to-back calls timed with "
                    "events, on the component-contiguous numbering of sc_reorder_csr (the solver's own)"}


def bench_kmeans(B, torch, args):
    """One step = one whole sc_kmeans call (seeding + Lloyd iterations to convergence) on points resident in HBM in
    the eigensolver's output layout.  Not the headline metric: a secondary line for the clustering step."""
    from paper_1802_04450_amd import workloads as wl
    if args.workload == "dti_like":     # the paper's largest clustering problem (Table "Datasets": 142,541 points, 500 clusters)
        import types
        cfg = types.SimpleNamespace(name="dti_like", n=142_541, k=500, seed=1802044500 + 31)
    else:
        cfg = wl.CONFIGS[int(args.workload.replace("cfg", ""))]
    n, k = cfg.n, cfg.k
    t0 = time.time()
    x = wl.embedding_like(n, k, cfg.seed + 100)
    log(f"[bench] k-means points: n={n}, d=k={k} in {time.time() - t0:.1f}s")
    pts = torch.as_tensor(np.ascontiguousarray(x.T), device="cuda")     # (d, n): column-major n x d
    seed, max_iter = 7, 100

    def run(timing=False):
        return B.sc_kmeans(pts, k, seed, max_iter, colmajor=True, timing=timing)

    for _ in range(max(1, args.warmup)):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        labels, cen, code, st = run(timing=True)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    out = {"metric": "k-means s (seeding + Lloyd to convergence) on the n x k embedding", "value": sec, "unit": "s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": f"kmeans on {cfg.name} embedding: n={n}, d={k}, k={k}, seed={seed}",
                      "status": int(code)},
           "kmeans_stats": st}
    if st["t_distance"] > 0:
        # per launch: points read once, product block written once (8 n (d + k) bytes), 2 n k d flops: 0.25 k d / (d + k)
        # flop per byte = 12.5 at d = k = 100, above the fp64 ridge of 9.8 flop/B: the matrix cores bound it
        tf = st["distance_flops"] / st["t_distance"] / 1e12
        out["roofline"] = {"bound": "mfma", "kernel": "row_gemm_kernel mode 1 (distance product V C^T, fp64 MFMA)",
                           "achieved": tf, "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": tf / FP64_MFMA_PEAK_TFLOPS, "traffic": None,
                           "launches_per_step": st["distance_launches"],
                           "avg_launch_us": st["t_distance"] / max(1, st["distance_launches"]) * 1e6,
                           "hbm_gbps_algorithmic": st["distance_bytes"] / st["t_distance"] / 1e9}
    if not args.no_cpu_baseline:
        from oracle import kmeans as okm
        ns = min(n, 20000)      # bounded sample: the first ns points, same k; the cost is linear in n
        t0 = time.time()
        _, _, iters, _, conv = okm.kmeans(x[:ns], k, seed, max_iter)
        dt = time.time() - t0
        try:
            import threadpoolctl
            threads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
        except Exception:
            threads = os.cpu_count() or 1
        out["cpu_baseline"] = {"value": dt * n / ns, "unit": "s", "cores": int(threads), "kind": "oracle",
                               "sample": f"oracle k-means on the first {ns} of {n} points took {dt:.2f}s "
                                         f"({iters} labelling steps); scaled by n/{ns}"}
    print(json.dumps(out), flush=True)


def bench_similarity(B, torch, args):
    """One step = cross-correlation similarity of every listed pair + symmetric CSR of the result, inputs resident in
    HBM.  Shape of the paper's DTI input (142,541 points of 90 coordinates, ~4.0 M neighbouring pairs)."""
    from paper_1802_04450_amd import workloads as wl
    n, d = 142_541, 90
    t0 = time.time()
    u, v = wl.voxel_neighbour_pairs(n)
    x = wl.connectivity_profiles(n, d, 1802044500 + 21)
    ne = int(u.size)
    log(f"[bench] similarity input: n={n}, d={d}, pairs={ne} in {time.time() - t0:.1f}s")
    dx = torch.as_tensor(x, device="cuda")
    du, dv = torch.as_tensor(u, device="cuda"), torch.as_tensor(v, device="cuda")

    def step():
        w = B.sc_edge_similarity(dx, du, dv, B.SC_SIM_CROSS_CORRELATION)
        return B.sc_coo_to_csr(du, dv, w, n, True)

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rp, co, vo = step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    # the similarity call alone, with events on the stream it runs on
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        B.sc_edge_similarity(dx, du, dv, B.SC_SIM_CROSS_CORRELATION)
    e1.record()
    torch.cuda.synchronize()
    t_sim = e0.elapsed_time(e1) * 1e-3 / reps
    # algorithmic bytes: the data once, the pair list, the values, the row statistics; what the kernel gathers is
    # 2 d 8 bytes per pair (5.7 GB here), served by the caches when neighbouring pairs share rows
    alg = 8.0 * n * d + 8.0 * ne + 8.0 * ne + 16.0 * n
    gathered = 16.0 * d * ne
    out = {"metric": "similarity graph s (Algorithm 1 cross correlation + COO to symmetric CSR)", "value": sec,
           "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": f"dti_like: n={n}, d={d}, pairs={ne}, nnz={int(rp[-1])}"},
           "roofline": {"bound": "hbm", "kernel": "row_stats_kernel + edge_similarity_kernel (one sc_edge_similarity call)",
                        "achieved": alg / t_sim / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": alg / t_sim / 1e9 / HBM_PEAK_GBS, "traffic": None, "call_us": t_sim * 1e6,
                        "gathered_gbps": gathered / t_sim / 1e9}}
    if not args.no_cpu_baseline:
        from oracle import similarity as osim
        ns = min(ne, 400_000)
        t0 = time.time()
        osim.edge_similarity(x, u[:ns], v[:ns], osim.CROSS_CORRELATION)
        dt = time.time() - t0
        out["cpu_baseline"] = {"value": dt * ne / ns, "unit": "s", "cores": 1, "kind": "oracle",
                               "sample": f"oracle cross correlation of the first {ns} of {ne} pairs took {dt:.2f}s; "
                                         f"scaled by pairs/{ns} (similarity only, no conversion)"}
    print(json.dumps(out), flush=True)


def bench_knn(B, torch, args):
    """One step = points -> exact k nearest neighbours -> undirected edge list with Gaussian weights -> symmetric CSR
    (Section III-A's k-nearest-neighbour graph), on the points of the benchmark workload, resident in HBM."""
    from paper_1802_04450_amd import workloads as wl
    key = int(args.workload[3:]) if args.workload.startswith("cfg") else 2
    cfg = wl.CONFIGS[key]
    x, _ = wl.mixture_points(cfg)
    n, d = x.shape
    k = cfg.k_nn
    dx = torch.as_tensor(x, device="cuda")

    def step():
        idx, dist = B.sc_knn_search(dx, k)
        sigma = float(dist.median())          # the workloads' bandwidth: the median neighbour distance
        eu, ev, w = B.sc_knn_union_pairs(idx, dist, sigma)
        return B.sc_coo_to_csr(eu, ev, w, n, True)

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rp, co, vo = step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(1, min(5, args.steps))
    e0.record()
    for _ in range(reps):
        B.sc_knn_search(dx, k)
    e1.record()
    torch.cuda.synchronize()
    t_knn = e0.elapsed_time(e1) * 1e-3 / reps
    # the search is a dense contraction (the cross term q.y of |q|^2 + |y|^2 - 2 q.y over all ordered pairs) on the
    # fp64 matrix cores, 2 n^2 d flops against their 78.6 TFLOP/s; the exact re-evaluation of the few candidates the
    # screen lets through is not counted
    flops = 2.0 * n * n * d
    out = {"metric": "kNN similarity graph s (exact k nearest neighbours + union edge list + symmetric CSR)",
           "value": sec, "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": f"{cfg.name} points: n={n}, d={d}, k_nn={k}, nnz={int(rp[-1])}"},
           "roofline": {"bound": "mfma", "kernel": "knn_mfma_kernel (one sc_knn_search call, with row padding and norms)",
                        "achieved": flops / t_knn / 1e12, "peak": 78.6, "unit": "TFLOP/s",
                        "frac": flops / t_knn / 1e12 / 78.6, "traffic": None, "call_ms": t_knn * 1e3}}
    if not args.no_cpu_baseline:
        from oracle import knn as oknn
        ns = max(2 * k, min(n, int(2.0e9 / (n * d))))       # queries whose n x d difference arrays take ~10-20 s
        t0 = time.time()
        ids = np.arange(n)
        for i in range(ns):                                   # the oracle's loop body on the first ns queries
            diff = x - x[i]
            d2 = (diff * diff).sum(axis=1)
            d2[i] = np.inf
            np.lexsort((ids, d2))[:k]
        dt = time.time() - t0
        out["cpu_baseline"] = {"value": dt * n / ns, "unit": "s", "cores": 1, "kind": "oracle",
                               "sample": f"the oracle's per-query search (all n distances, then the k smallest) for the "
                                         f"first {ns} of {n} queries took {dt:.2f}s; scaled by n/{ns} (search only)"}
    print(json.dumps(out), flush=True)


def timed_eigensolve(B, torch, cfg, dev, steps, warmup, block=0, m=None, check_every=0):
    """Survey solve (every kernel family event-timed, untimed by the wall clock), warm-ups, then `steps` solves timed
    with the wall clock between device synchronisations, HIP events round every launch of the dominant family only."""
    drp, dc, dv = dev
    kw = dict(m=cfg.m if m is None else m, block=block, check_every=check_every)

    def solve(timing_mask=0):
        return B.sc_laplacian_eigsh(drp, dc, dv, cfg.k, cfg.tol, timing_mask=timing_mask, **kw)

    survey = solve(timing_mask=63)[3]
    fam_t = survey["fam_time_s"]
    dom = int(np.argmax(fam_t))
    log(f"[bench] {cfg.name} kernel families (s per solve): "
        + ", ".join(f"{B.FAMILIES[f]}={fam_t[f]:.4f}" for f in range(6))
        + f"; host eig={survey['t_host_eig']:.4f}; total={survey['t_total']:.4f}")
    for _ in range(max(0, warmup - 1)):
        solve()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    last = None
    for _ in range(steps):
        last = solve(timing_mask=1 << dom)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    return sec, last, survey, dom


def family_rates(B, survey):
    out = {}
    for f in range(6):
        t = survey["fam_time_s"][f]
        if t > 0:
            out[B.FAMILIES[f]] = {"seconds_per_step": t, "launches": survey["fam_launches"][f],
                                  "hbm_gbps_algorithmic": survey["fam_bytes"][f] / t / 1e9,
                                  "hbm_frac": survey["fam_bytes"][f] / t / 1e9 / HBM_PEAK_GBS,
                                  "fp64_tflops": survey["fam_flops"][f] / t / 1e12,
                                  "fp64_mfma_frac": survey["fam_flops"][f] / t / 1e12 / FP64_MFMA_PEAK_TFLOPS}
    return out


def measured_ceilings(B, torch):
    """What the box itself reaches on the two resources the contraction kernels use, measured in this run: a plain
    device copy of 1 GiB (bytes read + written per second) and a launch that issues only fp64 matrix-core instructions.
    Context for the fractions of the published peaks, not a replacement for them."""
    src = torch.ones(1 << 27, dtype=torch.float64, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * src.numel() * 8 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()
    tf = max(B.sc_probe_fp64_matrix_rate(2048, 4000, 16) for _ in range(2))
    tf4 = max(B.sc_probe_fp64_matrix_rate(2048, 16000, 4) for _ in range(2))
    return {"copy_gbps_read_plus_write": copy_gbps, "copy_frac_of_hbm_peak": copy_gbps / HBM_PEAK_GBS,
            "fp64_mfma_only_tflops": tf, "fp64_mfma_only_frac_of_peak": tf / FP64_MFMA_PEAK_TFLOPS,
            "fp64_mfma_4x4x4_only_tflops": tf4, "fp64_mfma_4x4x4_only_frac_of_peak": tf4 / FP64_MFMA_PEAK_TFLOPS,
            "note": "fp64_mfma_only: the 16x16x4 form, which the contraction kernels use; the 4x4x4 form issues faster "
                    "but needs every operand value in the lanes of all blocks that use it"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=None,
                    help="cfg1..cfg5, syn200, dblp_like, fb_like; default cfg5 for the eigensolve, cfg2 for the secondary "
                         "stages (--kmeans, --knn)")
    ap.add_argument("--block", type=int, default=0)
    ap.add_argument("--m", type=int, default=-1)
    ap.add_argument("--check-every", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: no per_config solves of configs 1-3, no spmv_large, no complete "
                         "oracle run on config 2")
    ap.add_argument("--spmv-only", action="store_true",
                    help="build the workload, measure only the single-vector product y = S x, print its JSON and stop")
    ap.add_argument("--no-large-spmv", action="store_true",
                    help="skip the single-vector product on the 4,000,000-node workload (config 4) that the default run "
                         "adds as `spmv_large`: the product is bandwidth-bound only at that size (about 40 s, most of "
                         "it building the graph)")
    ap.add_argument("--kmeans", action="store_true",
                    help="the clustering step that follows the eigensolve (Algorithms 4-5) on a synthetic row-normalised "
                         "embedding of the workload's shape (n points, d = k; default config 2); prints its own JSON line")
    ap.add_argument("--similarity", action="store_true",
                    help="the graph-construction step (Algorithm 1 + the COO to CSR conversion of Algorithm 2) on "
                         "synthetic data of the shape of the paper's DTI input; prints its own JSON line")
    ap.add_argument("--knn", action="store_true",
                    help="the k-nearest-neighbour graph construction (Section III-A) on the points of --workload "
                         "(default config 2: n = 100,000, d = 32, k_nn = 20); prints its own JSON line")
    ap.add_argument("--ceilings", action="store_true",
                    help="only measure the practical ceilings the roofline fractions can be held against: a plain 1 GiB "
                         "device copy and a launch of nothing but fp64 matrix-core instructions")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain 1 GiB device copy 10 times (calibration of the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    if args.ceilings:
        from paper_1802_04450_amd import binding as B
        B.lib()
        print(json.dumps({"measured_ceilings": measured_ceilings(B, torch)}))
        return
    if args.copy_probe:
        src = torch.ones(1 << 27, dtype=torch.float64, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": src.numel() * 8, "copy_probe_bytes_written": src.numel() * 8}))
        return
    from paper_1802_04450_amd import binding as B
    B.lib()

    if args.workload is None:
        args.workload = "cfg2" if (args.kmeans or args.knn) else "cfg5"
    if args.kmeans:
        bench_kmeans(B, torch, args)
        return
    if args.similarity:
        bench_similarity(B, torch, args)
        return
    if args.knn:
        bench_knn(B, torch, args)
        return
    cfg, graph = build_workload(args.workload)
    rp, c, v, n = graph
    nnz = int(rp[-1])
    dev = B.csr_to_device(rp, c, v)
    if args.spmv_only:
        print(json.dumps({"workload": f"{cfg.name}: n={n}, nnz={nnz}", "spmv": measure_spmv(B, torch, *dev, n, nnz)}),
              flush=True)
        return
    sec, last, survey, dom = timed_eigensolve(B, torch, cfg, dev, args.steps, args.warmup, block=args.block,
                                              m=None if args.m < 0 else args.m, check_every=args.check_every)
    evals, evecs, code, stats = last
    fam_t = survey["fam_time_s"]
    spmv = measure_spmv(B, torch, *dev, n, nnz)

    out = {
        "metric": "eigensolve s + SpMV HBM GB/s, k smallest eigvecs of n-node kNN Laplacian",
        "value": sec, "unit": "s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={n}, nnz={nnz}, k={cfg.k}, m={stats['m']}, tol={cfg.tol}, "
                               f"block={stats['block']}", "status": int(code), "path": "plain (default options)"},
        "spmv": spmv,
        "solver_stats": stats,
    }
    kt = stats["fam_time_s"][dom]
    if kt > 0:
        launches = stats["fam_launches"][dom]
        ach = stats["fam_bytes"][dom] / kt / 1e9
        if args.block == 0 and args.m < 0:
            traffic, traffic_kernel, traffic_source, prof = profiled_traffic(args.workload, dom)
        else:
            traffic, traffic_kernel, traffic_source, prof = None, None, "non-default options", None
        # The counters are per kernel, the family's byte model averages over all of its launches (the long contractions
        # of traffic_kernel and many short ones of its sibling kernels), so the two per-launch figures are not of the same
        # launches.  For the two reorthogonalization GEMMs the profiled kernel's own algorithmic bytes follow from its
        # MFMA flop count: 2 n j b flops per launch give the contraction length j, the model 8 n (j + b) bytes for the
        # projection and 8 n (j + 2 b) for the update.
        traffic_alg = None
        if prof and prof["mfma_f64_flops_per_launch"] > 0 and dom in (1, 2):
            bb = stats["block"]
            j_avg = prof["mfma_f64_flops_per_launch"] / (2.0 * n * bb)
            traffic_alg = 8.0 * n * (j_avg + (1 if dom == 1 else 2) * bb)
        out["roofline"] = {"bound": "hbm", "kernel": KERNEL_OF_FAMILY[dom],
                           "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                           "traffic": traffic, "traffic_kernel": traffic_kernel, "traffic_source": traffic_source,
                           "traffic_kernel_algorithmic_bytes": traffic_alg,
                           "traffic_kernel_avg_us_profiled": prof["avg_launch_us_profiled"] if prof else None,
                           "launches_per_step": launches, "avg_launch_us": kt / max(1, launches) * 1e6,
                           "algorithmic_bytes_per_launch": stats["fam_bytes"][dom] / max(1, launches),
                           "fp64_tflops": stats["fam_flops"][dom] / kt / 1e12,
                           "fp64_mfma_frac": stats["fam_flops"][dom] / kt / 1e12 / FP64_MFMA_PEAK_TFLOPS,
                           "family_seconds_per_step": {B.FAMILIES[f]: fam_t[f] for f in range(6)},
                           "measured_ceilings": measured_ceilings(B, torch)}
    # every kernel family of the survey solve (all of them event-timed): achieved HBM rate by the byte model and fp64
    # rate against the matrix peak; "project" and "update" are the reorthogonalization GEMMs
    rates = family_rates(B, survey)
    out["families"] = rates
    out["reorth"] = {f: rates[f] for f in ("project", "update") if f in rates}
    if not args.no_cpu_baseline:
        if cfg.n <= 150_000:
            out["cpu_baseline"] = cpu_baseline_full(cfg, graph)
        else:
            out["cpu_baseline"] = cpu_baseline_extrapolated(cfg, graph)
    del dev, evals, evecs, last
    B.sc_release_cache()
    torch.cuda.empty_cache()

    if not args.no_extras:
        per = {}
        for name in ("cfg1", "cfg2", "cfg3"):
            if name == args.workload:
                continue
            cfg_x, graph_x = build_workload(name)
            dev_x = B.csr_to_device(*graph_x[:3])
            sec_x, last_x, survey_x, dom_x = timed_eigensolve(B, torch, cfg_x, dev_x, max(2, args.steps), 1)
            st = last_x[3]
            per[name] = {"workload": f"{cfg_x.name}: n={graph_x[3]}, nnz={int(graph_x[0][-1])}, k={cfg_x.k}, m={st['m']}, "
                                     f"tol={cfg_x.tol}, block={st['block']}",
                         "seconds": sec_x, "status": int(last_x[2]), "block_steps": st["block_steps"],
                         "filter_steps": st["filter_steps"], "spmv_cols": st["spmv_cols"], "phases": st["phases"],
                         "dominant_family": B.FAMILIES[dom_x], "families": family_rates(B, survey_x)}
            if name == "cfg2":
                per[name]["spmv"] = measure_spmv(B, torch, *dev_x, graph_x[3], int(graph_x[0][-1]))
                if not args.no_cpu_baseline:
                    out["cpu_baseline_cfg2"] = cpu_baseline_full(cfg_x, graph_x)
            del dev_x, last_x
            B.sc_release_cache()
            torch.cuda.empty_cache()
        out["per_config"] = per
        if not args.no_large_spmv and args.workload != "cfg4":
            # The product of the other workloads moves at most a few hundred MB and is latency bound; the HBM-bound figure
            # is the one of the 4,000,000-node workload, measured here in the same run (graph built on the box, resident
            # in HBM), on the numbering the solver works in.
            cfg4, graph4 = build_workload("cfg4")
            rp4, c4, v4, n4 = graph4
            nnz4 = int(rp4[-1])
            d4 = B.csr_to_device(rp4, c4, v4)
            large = measure_spmv(B, torch, d4[0], d4[1], d4[2], n4, nnz4)
            large["workload"] = f"{cfg4.name}: n={n4}, nnz={nnz4}"
            out["spmv_large"] = large
            del d4
            B.sc_release_cache()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
