/*
 * sceig - eigensolver for the symmetric normalized Laplacian of a sparse similarity graph,
 *         single AMD MI355X (gfx950), C ABI.
 *
 * Problem (paper Section II Steps 2-3, Section IV-B first paragraph): given a sparse symmetric
 * similarity matrix W (w_ij >= 0) with degrees D_ii = sum_j W_ij > 0 and a number k, return the k
 * eigenvectors belonging to the k smallest eigenvalues of the normalized Laplacian.  Section IV-B
 * switches to the k largest eigenvalues of the degree-normalized matrix; this library does the
 * same with the symmetric form S = D^-1/2 W D^-1/2 (similar to D^-1 W, so the eigenvalues are the
 * same) and reports lambda = 1 - theta for L = I - S.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory of the current device, owned by the caller; the library
 *     never frees or keeps them.  Inputs are const and never modified.  "host" pointers are ordinary
 *     host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work is
 *     enqueued on it; every call returns after that work has completed (stream synchronised).
 *   - Return value: 0 = SC_OK; > 0 = soft condition, outputs are valid as described; < 0 = error,
 *     outputs are unspecified.  No C++ exception crosses this boundary.
 *   - CSR: rowptr int64[n+1] with rowptr[0] = 0, non-decreasing, rowptr[n] = nnz; col int32[nnz] in
 *     [0, n); val fp64[nnz].  Columns need not be sorted; duplicate entries add up.  W must be
 *     symmetric with w_ij >= 0 (checked only under SC_FLAG_VALIDATE_SYMMETRY).  Self loops are allowed
 *     and count towards the degree.
 *   - Dense blocks handed to the kernel-level entry points are ROW-MAJOR: element (i, c) of an
 *     n x ncols block with leading dimension ld lives at base[i * ld + c].  The final eigenvector
 *     output of sc_laplacian_eigsh is COLUMN-MAJOR (vector t contiguous at evecs_out + t * n).
 *   - Calls that use the same stream or the same buffers must not overlap.
 *   - Workspace of a call is allocated inside it and cached between calls (see sc_release_cache()), except
 *     for sc_laplacian_eigsh_ws, which works inside a buffer of the caller's.
 */
#ifndef SCEIG_H
#define SCEIG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SC_OK 0
#define SC_NOT_CONVERGED 1 /* maxiter reached; outputs hold the best k Ritz pairs, stats->nconv met tol */
#define SC_EINVAL (-1)     /* null pointer, negative size */
#define SC_EDOMAIN (-2)    /* k < 1, k >= n, m out of range, block not supported, tol < 0 */
#define SC_ECSR (-3)       /* malformed CSR (rowptr not monotone, rowptr[0] != 0, column out of range); under
                              SC_FLAG_VALIDATE_SYMMETRY also an asymmetric W, a negative or a non-finite weight */
#define SC_EZERODEG (-4)   /* a row whose degree is <= 0 or not finite (Section IV-B: remove isolated nodes first) */
#define SC_ENOMEM (-5)     /* device or host allocation failed */
#define SC_EHIP (-6)       /* a HIP runtime call failed */
#define SC_EINTERNAL (-7)  /* an internal iteration limit was exceeded (the component pass did not settle) */

#define SC_FLAG_NO_VERIFY 1u /* skip the final deflated check phase (see sc_laplacian_eigsh) */
#define SC_FLAG_NO_REORDER 2u /* work on the CSR exactly as given: no connected-component pass, no internal
                                 renumbering of the nodes for gather locality */
#define SC_FLAG_COMPONENT_NULLSPACE 4u /* lock the closed-form eigenvalue-0 vectors D^1/2 1_C / sqrt(vol C) of the
                                 connected components (vol as in the Ncut definition of Section II) before the first
                                 Lanczos phase, after their residuals ||S v - v||, formed with block products, have met
                                 tol (if one does not, none is locked); off by default; ignored under SC_FLAG_NO_REORDER */

#define SC_FLAG_NO_START_FILTER 8u /* start every phase from the plain random block: no polynomial filtering of the
                                 re-injection blocks (see sc_laplacian_eigsh) */

#define SC_FLAG_FINAL_RR 16u /* always finish with a Rayleigh-Ritz step over the k locked vectors; by default that step
                                 only runs when some returned pair did not meet tol */

#define SC_FLAG_RANDOM_WALK_VECTORS 32u /* return u = D^-1/2 v, the eigenvectors of the paper's L_n = D^-1 L (Section II
                                 Steps 2-3), instead of the orthonormal v of the symmetric form: same eigenvalues,
                                 columns D-orthonormal (u_i^T D u_j = delta_ij), constant on every connected
                                 component for eigenvalue 0 */

#define SC_FLAG_ROW_NORMALIZE 64u /* scale every row of the n x k output (the k-dimensional embedding of a node that
                                 Section II Step 4 hands to k-means) to unit 2-norm; the columns are then no longer
                                 eigenvectors.  Applied after SC_FLAG_RANDOM_WALK_VECTORS, which it makes immaterial */

#define SC_FLAG_VALIDATE_SYMMETRY 128u /* check the precondition of the problem statement (Section II: W symmetric,
                                 w_ij >= 0) on the device before anything else: for every entry (i, j) the weights that row
                                 i lists under column j and row j under column i must add up to the same value (to four
                                 units in the last place), and every weight must be finite and >= 0; else SC_ECSR.  Costs
                                 one pass that reads two rows per entry */

/* Options; every field 0 = default. */
typedef struct sc_options {
  int32_t m;      /* budget of basis columns (locked + active Krylov vectors), the "number m of Lanczos
                     vectors" of Section IV-B; default min(n, max(2k, k + 56)); needs k + 3*block <= m <= n
                     (the library lowers `block` to fit when block is defaulted) */
  int32_t block;  /* Lanczos block size b in {1,2,4,8,16,32}; default 8 (n < 20,000), 16, or 32 (n >= 300,000 and k >= 1000),
                     lowered to fit k + 3b <= m and b <= next power of two >= k */
  int32_t check_every; /* block steps between convergence checks of the projected problem; default 2 */
  uint32_t flags; /* SC_FLAG_* */
  uint64_t seed;  /* seed of the start / re-injection blocks */
  uint32_t timing_mask; /* bit f set: time every launch of kernel family f with HIP events on the stream
                           (SC_FAM_*); results in sc_stats.fam_*; costs two event records per launch */
  int32_t guard;  /* extra pairs beyond k that the iteration converges and locks like the wanted ones (k + guard takes
                     the place of k in the defaults and limits of m and block); the k leading pairs are returned.  Makes
                     the k-th eigenvalue accurate to second order in tol when lambda_k and lambda_k+1 are close */
  const double* v0; /* device fp64[n], caller's numbering, finite, or NULL: start vector (Section IV-B notes that the
                     number of iterations varies with it); it becomes the first column of the first start block, the
                     other block - 1 columns and all later re-injection blocks are the seeded random ones */
} sc_options;

/* kernel families for timing_mask / sc_stats.fam_* */
#define SC_FAM_SPMM 0    /* sparse product with fused scaling */
#define SC_FAM_PROJECT 1 /* block projection H = Q^T W of the reorthogonalization (fp64 MFMA) */
#define SC_FAM_UPDATE 2  /* block update W -= Q H of the reorthogonalization (fp64 MFMA) */
#define SC_FAM_ROTATE 3  /* restart rotation / Ritz vectors V Y (fp64 MFMA) */
#define SC_FAM_QR 4      /* Cholesky QR of the new block (Gram, factorisation, scaling), per block step */
#define SC_FAM_OTHER 5   /* reductions of partial results */
#define SC_NUM_FAMILIES 6

typedef struct sc_stats {
  int32_t nconv;      /* wanted pairs whose residual estimate met tol */
  int32_t phases;     /* random (re-)starts */
  int32_t restarts;   /* thick restarts */
  int32_t block;      /* block size used */
  int32_t m;          /* basis budget used */
  int32_t host_eigs;  /* projected eigenproblems solved on the host */
  int32_t components; /* connected components found by the setup pass (0 under SC_FLAG_NO_REORDER) */
  int32_t filter_steps; /* block products spent on Chebyshev filtering of start blocks (counted in spmv_cols too) */
  int64_t block_steps;
  int64_t spmv_cols;  /* columns multiplied by S in total */
  double t_total;     /* seconds, whole call */
  double t_host_eig;  /* seconds in the host projected eigenproblems */
  double t_setup;     /* seconds: validation, degrees, allocation */
  double max_residual_est; /* largest residual estimate among the returned pairs */
  /* per kernel family, only for the families selected in sc_options.timing_mask: */
  double fam_time_s[6];   /* summed launch durations (HIP events) */
  double fam_bytes[6];    /* summed algorithmic bytes of those launches */
  double fam_flops[6];    /* summed algorithmic flops of those launches */
  int64_t fam_launches[6];
} sc_stats;

/*
 * The hot path (Algorithm 3 re-designed GPU-resident): k smallest eigenpairs of
 * L = I - D^-1/2 W D^-1/2, counted with multiplicity.
 *
 *   csr_rowptr, csr_col, csr_val  device, CSR of W as described above
 *   n, k                          1 <= k < n
 *   tol                           a Ritz pair counts as converged when its residual estimate
 *                                 ||S x - theta x||_2 <= tol   (||S||_2 = 1); tol >= 0
 *   maxiter                       upper bound on restart cycles (phase starts + thick restarts); >= 1
 *   evals_out                     device, fp64[k], ascending eigenvalues of L
 *   evecs_out                     device, fp64[n*k], column-major, orthonormal eigenvectors of L
 *                                 (v = D^1/2 u for the eigenvectors u of the paper's D^-1 L; u itself under
 *                                 SC_FLAG_RANDOM_WALK_VECTORS)
 *   opt, stats                    host, may be NULL
 *
 * Method: block Lanczos with full reorthogonalization (classical Gram-Schmidt, first pass against all
 * locked and active basis vectors, second pass against the active Krylov vectors; a phase's random start
 * block gets both passes against everything), thick restart, locking, and re-injection of a fresh random
 * block after every lock so that multiple eigenvalues are found with their multiplicity; once k pairs
 * are locked one further deflated phase must find nothing better (skipped under SC_FLAG_NO_VERIFY, and when
 * the k-th locked theta is already within tol of 1, the largest value the spectrum of S can reach for W >= 0);
 * the outputs are the locked Ritz pairs in ascending order of lambda (after a Rayleigh-Ritz step over them when
 * some pair did not meet tol, or under SC_FLAG_FINAL_RR).  Only the projected
 * eigenproblems (size <= m) run on the host.
 *
 * Returns SC_OK, SC_NOT_CONVERGED, or an error (< 0).
 */
int sc_laplacian_eigsh(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n, int32_t k,
                       double tol, int32_t maxiter, double* evals_out, double* evecs_out, void* stream,
                       const sc_options* opt, sc_stats* stats);

/*
 * Device memory, in bytes, that sc_laplacian_eigsh takes for itself for a problem of this size (an upper estimate of the
 * sum of its blocks: its renumbered copy of the operator, the basis n x (m + b), the rotation workspace, the packed
 * block, partial-sum and coefficient buffers), with the same defaults for opt->m and opt->block as the solve (opt->flags
 * and opt->guard count too).  Nothing is allocated and no GPU is needed.  This is also the size of the buffer that
 * sc_laplacian_eigsh_ws needs.
 *   bytes_out  host
 * Returns SC_OK, SC_EINVAL, or SC_EDOMAIN exactly where the solve would.
 */
int sc_workspace_bytes(int64_t n, int64_t nnz, int32_t k, const sc_options* opt, size_t* bytes_out);

/*
 * sc_laplacian_eigsh (same problem statement: Section II Steps 2-3, Section IV-B) with every device block of the solve
 * carved out of a buffer that the caller owns, so that the caller's allocator (PyTorch's, say) accounts for all device
 * memory: the call makes no device allocation and does not touch the library's block cache.
 *   workspace        device, at least sc_workspace_bytes(n, nnz, k, opt) bytes (nnz = csr_rowptr[n]); any alignment
 *                    (up to 255 bytes are skipped to reach a 256-byte boundary; the estimate allows for that);
 *                    contents on entry are ignored, on return unspecified
 *   workspace_bytes  its size; SC_ENOMEM if it is smaller than the estimate (nothing has been computed then)
 * Everything else as sc_laplacian_eigsh, results bitwise equal to it for equal arguments.  A few KB of pinned host
 * memory (coefficient blocks read back during convergence checks) still come from the library's own pinned cache.
 */
int sc_laplacian_eigsh_ws(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n, int32_t k,
                          double tol, int32_t maxiter, double* evals_out, double* evecs_out, void* stream,
                          const sc_options* opt, sc_stats* stats, void* workspace, size_t workspace_bytes);

/*
 * Setup step (Algorithm 2 steps 1-2, with the scaling kept as a vector instead of a scaled copy of W):
 * d_i = sum_j W_ij and s_i = d_i^-1/2.   d_out, s_out: device fp64[n] (d_out may be NULL).
 * Returns SC_EZERODEG if some d_i is <= 0 or not finite (outputs then hold what was computed).
 */
int sc_degree_scaling(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                      double* d_out, double* s_out, void* stream);

/*
 * The sparse product of Algorithm 3's loop body with the degree scaling fused in:
 *   Y = diag(s) W diag(s) X   for an n x ncols block, ncols in {1,2,4,8,16,32}.
 *   s     device fp64[n] (from sc_degree_scaling); or NULL: csr_val then holds the scaled operator S_ij = s_i W_ij s_j
 *         (from sc_scale_operator, the materialised form of Algorithm 2 step 3) and Y = S X is one launch with no
 *         scaling pass; x is gathered in place when it is packed (ldx == ncols) and 16-byte aligned
 *   x     device, row-major n x ncols, leading dimension ldx >= ncols
 *   y     device, row-major n x ncols, leading dimension ldy >= ncols; must not alias x
 *   work  device fp64[n*ncols] scratch (holds diag(s) X packed), 16-byte aligned (else SC_EINVAL); may be NULL,
 *         then it is allocated and freed inside the call (nothing is needed when x is gathered in place)
 * Exception to the general rule: when `work` is given, or x is gathered in place, this call only ENQUEUES on `stream`
 * and returns without synchronising (products can be issued back to back); else it returns after completion.
 * CSR columns are NOT range-checked here (sc_validate_csr does that).
 */
int sc_spmm_normalized(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                       int64_t n, const double* x, int64_t ldx, double* y, int64_t ldy, int32_t ncols, double* work,
                       void* stream);

/*
 * The single-vector product of Algorithm 3's loop body as it occurs in a chain of products (a Lanczos or power
 * iteration), with the degree scaling fused on both sides and no pass of its own for it: the operand arrives scaled,
 * z_in = s o x (elementwise), as the previous product left it, and the call produces in ONE launch
 *   y = s o (W z_in)  ( = diag(s) W diag(s) x )   and   z_out = s o y, the operand of the next product.
 * The first operand of a chain is formed by the caller (z = s o x, any elementwise multiply).
 *   s, z_in   device fp64[n];  y, z_out  device fp64[n], neither may be z_in
 *   nnz       csr_rowptr[n], passed by the caller (it only steers the choice of the tile shape)
 * ENQUEUES on `stream` and returns without synchronising, so that products can be issued back to back.
 * CSR columns are NOT range-checked here (sc_validate_csr does that).
 */
int sc_spmv_normalized_chain(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                             int64_t n, int64_t nnz, const double* z_in, double* y, double* z_out, void* stream);

/*
 * Algorithm 2 step 3 (ScaleElements) in its symmetric form: val_out[e] = s_i * csr_val[e] * s_j for entry e = (i, j).
 * The two factors are applied in index order, so (i, j) and (j, i) get the same rounding and the copy is exactly
 * symmetric when W is.  val_out (device fp64[nnz]) may be csr_val itself.
 */
int sc_scale_operator(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                      int64_t n, double* val_out, void* stream);

/*
 * The setup pass sc_laplacian_eigsh runs unless SC_FLAG_NO_REORDER is set, as a step of its own: connected
 * components of W (entries with weight exactly 0 do not connect) by label propagation on the device, and the
 * component-contiguous renumbering of the nodes; inside a component nodes are ordered by three levels of
 * neighbourhood min-hash (nodes that share neighbours become neighbours; a deterministic function of the graph).
 * The solver itself, when it works with blocks of 8 or more vectors on a graph with hubs (longest row more than
 * three average rows), puts the row length before the min-hash levels; this call never does.
 *   rowptr_out int64[n+1], col_out int32[nnz], val_out fp64[nnz]   device, the renumbered CSR
 *   old_of_new_out int32[n]   device: original index of new node p (y_orig[old_of_new[p]] = y_new[p])
 *   ncomp_out                 host, number of connected components (may be NULL)
 * The CSR is validated first (SC_ECSR).
 */
int sc_reorder_csr(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                   int64_t* rowptr_out, int32_t* col_out, double* val_out, int32_t* old_of_new_out, int32_t* ncomp_out,
                   void* stream);

/* Structural check of a device CSR: SC_OK or SC_ECSR. */
int sc_validate_csr(const int64_t* csr_rowptr, const int32_t* csr_col, int64_t n, void* stream);

/*
 * The start-block filter of sc_laplacian_eigsh as a step of its own (the start vector of Algorithm 3 is free; the
 * solver passes its re-injection blocks through this polynomial):
 *   Y = T_d(g(S)) X,   T_d = Chebyshev polynomial of the first kind of degree d,
 *   g(S) = (2 S - (a - 1) I) / (a + 1), the affine map that takes the interval [-1, a] of the spectrum to [-1, 1],
 * by the three-term recurrence Y_0 = X, Y_1 = g(S) X, Y_{i+1} = 2 g(S) Y_i - Y_{i-1}: d sparse products, nothing else.
 * An eigenvector of S with eigenvalue theta is multiplied by T_d((2 theta - a + 1) / (a + 1)): at most 1 in modulus
 * for theta in [-1, a], cosh(d acosh(.)) above a.
 *   x, y    device, row-major n x ncols with leading dimensions ldx, ldy >= ncols; ncols in {1,2,4,8,16,32}; y may be x
 *   a       -1 < a < 1;  degree >= 1
 * For ncols >= 8 the products run on a scaled copy of the operator made inside the call (as the solver does), for
 * narrower blocks on W and the scaling vector.  When the matrix as given is block diagonal (contiguous diagonal blocks,
 * e.g. one per connected component) with blocks small enough for two iterates of at least two columns to fit the LDS of
 * a compute unit, and a cost model favours it, the ncols >= 8 filter runs as ONE launch in which a workgroup keeps the
 * iterates of its block in LDS through all d steps; otherwise as d launches of the product kernel.  Both give the
 * recurrence's result to rounding; each is bitwise reproducible.  Returns SC_EZERODEG if some degree is not positive.
 */
int sc_chebyshev_filter(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                        const double* x, int64_t ldx, int32_t ncols, double a, int32_t degree, double* y, int64_t ldy,
                        void* stream);

/*
 * One reorthogonalization of the Lanczos recurrence (inside TakeStep of Algorithm 3): classical
 * Gram-Schmidt applied twice to the block W = basis[:, j : j+b] against Q = basis[:, 0 : j]:
 *   H1 = Q^T W, W -= Q H1, H2 = Q^T W, W -= Q H2, h_out = H1 + H2.
 *   basis  device, row-major n x ld, ld >= j + b; columns j..j+b-1 are updated in place
 *   h_out     device fp64[j*b], row-major j x b (may be NULL)
 *   gram_out  device fp64[b*b], row-major: W^T W of the updated block, accumulated in the same pass as the
 *             second update (this is the Gram matrix the block orthonormalization starts from); may be NULL
 *   1 <= b <= 32, j >= 0 (j = 0: nothing is done, outputs untouched).
 */
int sc_cgs2(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* h_out, double* gram_out,
            void* stream);

/*
 * Orthonormalization of the block W = basis[:, j : j+b] by Cholesky QR applied twice: W = Q R.
 * Columns that are numerically dependent on the columns before them (or zero) become exactly
 * zero columns of Q and zero rows of R.
 *   r_out  device fp64[b*b] row-major upper triangular R (may be NULL)
 *   g_out  device fp64[b*b] Gram matrix W^T W of the block before orthonormalization (may be NULL)
 */
int sc_block_qr(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* r_out, double* g_out,
                void* stream);

/*
 * sc_block_qr for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same arithmetic and same results as sc_block_qr, but the call allocates nothing
 * (no hipMalloc / hipFree, no block cache): its partial Gram blocks and small matrices live in a fixed device array of
 * 12.6 MB inside the library (about 1.58 million doubles), which every GPU the library runs on holds from the first such
 * call on it until the process ends.
 *   Limits: b in {1,2,4,8,16,32} (the array is sized for 32 columns; the number of partial blocks does not grow with
 *   n), n <= 2^31 - 1; anything else is SC_EDOMAIN and nothing is written.
 *   All calls on one GPU share that one array: calls that overlap in time on the same GPU (from several threads or
 *   streams) race and give undefined results; serialise them.  Nothing in the array has to be cleared between calls
 *   (every entry is written before it is read), and its contents after a call are unspecified.
 * Returns after the work on `stream` is done, like sc_block_qr.
 */
int sc_block_qr_noalloc(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* r_out, double* g_out,
                        void* stream);

/*
 * Restart rotation / Ritz vectors (FindEigenvectors of Algorithm 3): out = basis[:, j0 : j0+ja] * Y.
 *   y       device fp64[ja*l], row-major ja x l
 *   out     device; if out_colmajor == 0 row-major n x l with leading dimension ldo >= l,
 *           else column-major (column t contiguous at out + t*ldo, ldo >= n); must not alias basis
 */
int sc_rotate(const double* basis, int64_t n, int64_t ld, int32_t j0, int32_t ja, const double* y, int32_t l,
              double* out, int64_t ldo, int32_t out_colmajor, void* stream);

/*
 * Projected eigenproblem (the m x m eigendecomposition of Section IV-B), HOST ONLY, no GPU needed:
 * all eigenpairs of a dense symmetric matrix.
 *   a     host fp64[n*n], symmetric, row-major (only read)
 *   w     host fp64[n], eigenvalues ascending
 *   z     host fp64[n*n], row-major, column t (z[i*n+t]) is the eigenvector of w[t]; may be NULL
 * Returns SC_OK, SC_EINVAL, SC_ENOMEM, or SC_NOT_CONVERGED if the QL iteration failed.
 */
int sc_sym_eig(const double* a, int32_t n, double* w, double* z);

/*
 * The same projected eigenproblem when only the leading Ritz vectors are needed (convergence checks, locking,
 * thick restart): all eigenvalues, eigenvectors of the `count` largest only.  HOST ONLY.
 *   w     host fp64[n], eigenvalues ascending
 *   z     host fp64[n*count], row-major n x count; column t is the eigenvector of w[n-1-t]
 *   0 <= count <= n
 */
int sc_sym_eig_top(const double* a, int32_t n, int32_t count, double* w, double* z);

/*
 * k-means on the rows of the eigenvector matrix (Section II Step 4; Section IV-C, Algorithms 4 and 5).
 *
 * Points: n points with d coordinates, device fp64, read only.  colmajor != 0: coordinate t of point i at
 * points[t*ld + i], ld >= n (the evecs_out layout of sc_laplacian_eigsh, so its output can be passed on as it is);
 * colmajor == 0: points[i*ld + t], ld >= d.  Centres: device fp64[k*d], row-major k x d.  Labels: device int32[n].
 * 1 <= k <= n <= 2^27, d >= 1 (else SC_EDOMAIN).  All work is enqueued on `stream`; the calls return after it is done.
 * The library stages its own row-major copy of the points and never keeps a caller's pointer.
 */
typedef struct sc_kmeans_stats {
  int32_t iterations;   /* labelling steps done */
  int32_t converged;    /* 1 if the last labelling step changed no label */
  int32_t last_changes; /* labels changed by the last labelling step */
  int32_t timing;       /* INPUT: nonzero = bracket every distance-product launch with events on the stream and
                           report their summed duration below (the only field read on entry; all others are outputs) */
  double objective;     /* sum of squared distances of the points to the centres of their labels; -1 if the run stopped
                           at max_iter (the centres moved after the last labelling) */
  double t_total;       /* seconds, host clock, whole call */
  double t_seed;        /* seconds spent in the seeding */
  double t_distance;    /* seconds, device clock, all distance-product launches (V C^T); 0 unless timing was set */
  int64_t distance_launches;
  double distance_bytes; /* algorithmic bytes of those launches: points read + product block written + centres */
  double distance_flops; /* 2 n k d per labelling step */
} sc_kmeans_stats;

/*
 * Seeding (Algorithm 5): the first centre is the point floor(u_0 * n); centre i > 0 is drawn with probability
 * proportional to the squared distance to the nearest centre chosen so far: the first index whose inclusive prefix
 * sum of those squared distances exceeds u_i * (their total); the last point if no index does.  u_i is the i-th
 * number of a counter-based generator: the top 53 bits of mix(mix(seed) + i) scaled to [0, 1), mix being the
 * splitmix64 output function (add 0x9E3779B97F4A7C15, xor-shift 30, multiply 0xBF58476D1CE4E5B9, xor-shift 27,
 * multiply 0x94D049BB133111EB, xor-shift 31).
 *   chosen_out     device int32[k], indices of the chosen points in drawing order (may be NULL)
 *   centroids_out  device fp64[k*d], the chosen points
 */
int sc_kmeanspp(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k, uint64_t seed,
                int32_t* chosen_out, double* centroids_out, void* stream);

/*
 * Lloyd iterations (Algorithm 4 step 3) from the centres given in `centroids`, which are updated in place.
 * One iteration: label of every point = the nearest centre, decided on |c_j|^2 - 2 <v_i, c_j> (the expanded form of
 * Section IV-C with the product V C^T on the fp64 matrix cores; the lowest index wins a tie); stop if no label
 * changed; else every centre becomes the mean of its points (points grouped by a sort on the labels; a centre without
 * points stays where it is).  At most max_iter (>= 1) labelling steps.
 * Returns SC_OK, or SC_NOT_CONVERGED if labels still changed in the last step (outputs hold the last labels and the
 * centres computed from them).
 */
int sc_kmeans_lloyd(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k,
                    double* centroids, int32_t max_iter, int32_t* labels_out, sc_kmeans_stats* stats, void* stream);

/* Algorithm 4: sc_kmeanspp followed by sc_kmeans_lloyd. */
int sc_kmeans(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k, uint64_t seed,
              int32_t max_iter, int32_t* labels_out, double* centroids_out, sc_kmeans_stats* stats, void* stream);

/*
 * Similarity of the listed pairs of data points (Section IV-A; Algorithm 1 steps 4-6).
 *   x        device fp64, n x d row-major with leading dimension ldx >= d (read only: the centring of Algorithm 1 step 5
 *            is applied on the fly, the caller's data are not modified)
 *   edge_u, edge_v  device int32[nedges]: the pairs (the paper's list E of neighbouring points)
 *   measure  SC_SIM_CROSS_CORRELATION: <x_u - mean(x_u), x_v - mean(x_v)> / (|x_u - mean(x_u)| |x_v - mean(x_v)|)
 *            SC_SIM_COSINE:            <x_u, x_v> / (|x_u| |x_v|)
 *            SC_SIM_EXP_DECAY:         exp(-|x_u - x_v|^2 / (2 sigma^2)), sigma > 0 (the paper prints this measure
 *                                      without the minus sign and the square; a similarity has both)
 *   val_out  device fp64[nedges]; a constant row gives NaN under the first two measures (0/0), as the definition does
 * Returns SC_ECSR if an index is outside [0, n) (that edge's value is NaN, no row was read for it), SC_EDOMAIN for
 * d < 1, ldx < d, an unknown measure or sigma <= 0.
 */
#define SC_SIM_CROSS_CORRELATION 0
#define SC_SIM_COSINE 1
#define SC_SIM_EXP_DECAY 2
int sc_edge_similarity(const double* x, int64_t ldx, int64_t n, int32_t d, const int32_t* edge_u, const int32_t* edge_v,
                       int64_t nedges, int32_t measure, double sigma, double* val_out, void* stream);

/*
 * k-nearest-neighbour search for the k-nearest-neighbour similarity graph (Section III-A: x_i and x_j are connected
 * if either is among the k nearest of the other; k_nn is unrelated to the number of clusters).  Exact, by Euclidean
 * distance, brute force: the squared distance is the plain sum of squared coordinate differences in fp64.
 *   x         device fp64, n x d row-major with leading dimension ldx >= d (read only)
 *   idx_out   device int32[n * k_nn]: row i = the k_nn points nearest to x_i other than i, nearest first; equal
 *             distances are ordered by index, so the result is unique
 *   dist_out  device fp64[n * k_nn]: their Euclidean distances
 * 2 <= n <= 2^31 - 1, d >= 1, 1 <= k_nn <= n - 1, and the kernel's LDS need must fit a workgroup's 160 KB, else
 * SC_EDOMAIN: 768 * k_nn + 1536 bytes for d <= 128 (any k_nn up to 200), 128 * (8 * dp + 12 * k_nn) bytes for d > 128
 * (dp = d rounded up to a multiple of 8).  The library allocates n * (dp + 1) * 8 bytes of scratch for the call, dp = d
 * rounded up to 8, 16, 32, 64 or 128 (to a multiple of 8 beyond).  Returns after the work on `stream` is done.
 */
int sc_knn_search(const double* x, int64_t ldx, int64_t n, int32_t d, int32_t k_nn, int32_t* idx_out, double* dist_out,
                  void* stream);

/*
 * The undirected edges of the k-nearest-neighbour graph (Section III-A's "either ... or": the union of the directed
 * neighbour relation), each once, in the form sc_coo_to_csr takes with symmetrize = 1.
 *   idx, dist  device, n x k_nn neighbour lists as sc_knn_search writes them (entries < 0 or >= n and i's own index
 *              are skipped, a neighbour listed twice in a row counts once)
 *   sigma      0: val = the listed distance; > 0: val = exp(-dist^2 / (2 sigma^2)), the Gaussian weight of Section
 *              IV-A (weights that underflow to 0 are kept: dropping them is the caller's choice)
 *   edge_u, edge_v, val_out  device, room for n * k_nn entries; the first *npairs_out are the edges with
 *              edge_u < edge_v, grouped by the row whose list emitted them (the lower index, or the higher one if
 *              only its list holds the pair), in list order; what lies beyond is unspecified
 *   npairs_out host
 * n * k_nn <= 2^31 - 1, k_nn >= 1, sigma >= 0 (else SC_EDOMAIN).
 */
int sc_knn_union_pairs(const int32_t* idx, const double* dist, int64_t n, int32_t k_nn, double sigma, int32_t* edge_u,
                       int32_t* edge_v, double* val_out, int64_t* npairs_out, void* stream);

/*
 * Coordinate format to CSR (Algorithm 2 step 4), on the device.
 *   row, col, val   device, nnz_in entries (r, c, w) in any order
 *   symmetrize      nonzero: every listed entry with r != c also stands for (c, r, w) - the list names each undirected
 *                   edge once, as Algorithm 1's pair list does
 *   rowptr_out      device int64[n+1]
 *   col_out, val_out  device, room for nnz_in * (symmetrize ? 2 : 1) entries; the first rowptr_out[n] are the matrix,
 *                   sorted by (row, col); entries listed more than once stay separate (the products add them up) in
 *                   listing order; what lies beyond rowptr_out[n] is unspecified
 *   nnz_out         host, = rowptr_out[n]; may be NULL
 * n <= 2^31 - 1 and at most 2^31 - 1 output entries (else SC_EDOMAIN); SC_ECSR if an index is outside [0, n).
 */
int sc_coo_to_csr(const int32_t* row, const int32_t* col, const double* val, int64_t nnz_in, int64_t n,
                  int32_t symmetrize, int64_t* rowptr_out, int32_t* col_out, double* val_out, int64_t* nnz_out,
                  void* stream);

const char* sc_strerror(int code);
int sc_version(void);

/*
 * Process-wide event counters (for tests and tuning: which code path a call took).  HOST ONLY.
 *   SC_COUNTER_RESIDENT_FILTERS  start-block filters (inside sc_laplacian_eigsh or sc_chebyshev_filter) that ran as one
 *                                launch with the iterates resident in LDS, since the library was loaded
 * Returns the count, or -1 for an unknown id.
 */
#define SC_COUNTER_RESIDENT_FILTERS 0
int64_t sc_counter(int32_t which);

/*
 * Measurement aid (Section V reports rates against the hardware's peaks; this gives the practical one for the fp64
 * matrix cores, which the reorthogonalization, rotation, distance-product and neighbour-search kernels run on).
 * Launches `workgroups` workgroups of four waves that issue nothing but fp64 matrix instructions (iterations * 8 per
 * wave, eight independent accumulators) on `stream`, times the launch with events and stores the rate in TFLOP/s.
 *   shape       16: the 16x16x4 form (2,048 flops per instruction; the form the library's kernels use),
 *               4: the 4x4x4 form (four independent 4x4 blocks, 512 flops per instruction); else SC_EDOMAIN
 *   tflops_out  HOST pointer
 *   1 <= workgroups <= 2^20, 1 <= iterations <= 2^24 (else SC_EDOMAIN); the call synchronizes the stream.
 */
int sc_probe_fp64_matrix_rate(int32_t shape, int32_t workgroups, int32_t iterations, double* tflops_out, void* stream);

/*
 * Memory.  Device and pinned-host blocks that a call allocates for itself are kept by the library when the call
 * returns and handed to later calls that ask for a block of exactly the same size on the same device (a repeated
 * solve of one problem shape then allocates nothing).  At most 4 GiB of device memory (and as much pinned memory)
 * are held this way; the environment variable SCEIG_CACHE_LIMIT_MB, read once, sets another limit, 0 switches the
 * caching off.  sc_release_cache() gives everything held back to the HIP runtime; call it only while no other call
 * into the library is running.  Returns SC_OK.
 */
int sc_release_cache(void);

#ifdef __cplusplus
}
#endif
#endif /* SCEIG_H */
