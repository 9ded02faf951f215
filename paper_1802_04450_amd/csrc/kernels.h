// Launch wrappers of the gfx950 kernels.  All pointers are device pointers unless said otherwise;
// every wrapper only enqueues work on `st` and returns hipGetLastError().
//
// Dense blocks are row-major: element (i, c) of a block with leading dimension ld is p[i*ld + c].
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sceig {

constexpr int kMaxBlock = 32;      // largest Lanczos block size
constexpr int kLongRow = 128;      // rows with more entries than this are "long" for the wide sparse products
constexpr int kPartialPad = 32;    // column stride of partial / coefficient blocks (>= kMaxBlock)

// ---- setup ---------------------------------------------------------------------------------
// flag[0] |= 1 if rowptr is not monotone / rowptr[0] != 0, |= 2 if a column is out of range.
hipError_t launch_validate_csr(const int64_t* rowptr, const int32_t* col, int64_t n, int64_t nnz, int* flag,
                               hipStream_t st);
// flag[0] |= 8 if W is not symmetric (for some entry (i, j) the weights listed in row i under column j and in row j
// under column i add up to different values), |= 16 if a weight is negative or not finite.  Only for a CSR that
// launch_validate_csr has accepted (columns are used as row indices).
hipError_t launch_validate_symmetry(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, int* flag,
                                    hipStream_t st);
// d_i = sum of row i, s_i = d_i^-1/2; flag[0] |= 4 if some d_i is <= 0 or not finite.  d may be null.
hipError_t launch_degree_scaling(const int64_t* rowptr, const double* val, int64_t n, double* d, double* s, int* flag,
                                 hipStream_t st);

// ---- sparse product ------------------------------------------------------------------------
// z[i*b + t] = s[i] * x[i*ldx + t]   (packed scaled copy of an n x b block)
hipError_t launch_pack_scaled(const double* x, int64_t ldx, const double* s, int64_t n, int b, double* z,
                              hipStream_t st);
// y[i*ldy + t] = s[i] * sum_e val[e] * z[col[e]*b + t]  over the entries e of row i; b in {1,2,4,8,16,32}.
// s == null: no row scaling (the values are the scaled operator S_ij and z = x).
// avg_deg steers the lanes-per-row choice of the b <= 4 kernels.
hipError_t launch_spmm(const int64_t* rowptr, const int32_t* col, const double* val, const double* s, int64_t n,
                       const double* z, int b, double* y, int64_t ldy, double avg_deg, hipStream_t st);

// Single-vector product inside a chain of products: z = s o x (the operand, scaled by the call that produced x),
// y = s o (W z), zout = s o y (the operand of the next product), one launch.
hipError_t launch_spmv_chain(const int64_t* rowptr, const int32_t* col, const double* val, const double* s, int64_t n,
                             const double* z, double* y, double* zout, double avg_deg, hipStream_t st);

// ---- tall-skinny projections (fp64 MFMA) ---------------------------------------------------
struct ProjectPlan {
  int rows_per_panel;  // multiple of 4
  int nwc;             // waves of a workgroup laid along the columns (1, 2 or 4)
  int npart;           // number of partial blocks produced = row panels (one per workgroup: waves that share a
                       // column tile add their sums inside the workgroup)
};
ProjectPlan plan_project(int64_t n, int ja, int max_partials);
// part[p][c][t] (c < ja, t < kPartialPad) = sum over the rows of partial p of A[i, acol0 + c] * B[i, bcol0 + t]
// with A and B both columns of `basis` (row-major n x ld); t >= b entries are written as 0.
// skip (here and below; may be null): device int; if *skip != 0 when the kernel starts, the launch does nothing.
hipError_t launch_project(const double* basis, int64_t n, int64_t ld, int acol0, int ja, int bcol0, int b,
                          const ProjectPlan& plan, double* part, hipStream_t st, const int* skip = nullptr);
// h[c*kPartialPad + t] = sum_p part[p][c][t] in the fixed order p = 0..npart-1 (t < b, else 0);
// if hsum != null: hsum = (accumulate ? hsum : 0) + h.
// if slot != null: rows [slot_row0, ja) of the resulting hsum (or h) are copied to slot[(c-slot_row0)*kPartialPad + t].
hipError_t launch_reduce_partials(const double* part, int npart, int ja, int b, double* h, double* hsum,
                                  int accumulate, double* slot, int slot_row0, hipStream_t st,
                                  const int* skip = nullptr);
// skip[0] = 1 when no column of the block needs a second Gram-Schmidt pass: for every column t < b the squared norm
// the first pass removed, sum_c h[c*kPartialPad + t]^2 over c < ja, is at most ratio2 times the squared norm it kept,
// gram[t*kPartialPad + t]; else skip[0] = 0.
hipError_t launch_second_pass_test(const double* h, int ja, int b, const double* gram, double ratio2, int* skip,
                                   hipStream_t st);

// C = A * B row GEMM:  A = basis[:, acol0 : acol0+kdim] (n x kdim), B = bmat (kdim x ncols, row-major, ldb).
// mode 0: basis[:, ccol0 + t] -= C[:, t]          (in place update, ncols <= 32, out unused)
// mode 1: out[i*ldo + t]  = C[i, t]                (row-major)
// mode 2: out[t*ldo + r(i)] = C[i, t]             (column-major; r(i) = rowmap[i] if rowmap != null, else i)
// mode 3: basis[:, ccol0 + t] = C[:, t]           (ncols <= 64, out unused; the columns written may be among the
//         columns read: one wave owns all ncols entries of its rows and stores them after its last read of those rows)
hipError_t launch_row_gemm(double* basis, int64_t n, int64_t ld, int acol0, int kdim, const double* bmat, int ldb,
                           int ncols, int mode, int ccol0, double* out, int64_t ldo, const int32_t* rowmap,
                           hipStream_t st, const int* skip = nullptr);

// ---- block orthonormalization --------------------------------------------------------------
// One Cholesky-QR pass bookkeeping on the Gram matrix g_in (b x b, stride kPartialPad; single workgroup):
//   Cholesky g = r^T r with dependent columns dropped (zero row in r, zero row+column in rinv);
//   rinv = r^-1 on the kept columns; g_out = symmetrised copy of g_in.
//   If rprev != null: rout = r * rprev (composition of two passes) else rout = r.  Any output may be null.
hipError_t launch_gram_cholesky(const double* g_in, int b, double* g_out, double* rinv, double* rout,
                                const double* rprev, double abs_tol2, double rel_tol, hipStream_t st);
// basis[:, col0 : col0+b] = basis[:, col0 : col0+b] * rinv  (rinv b x b row-major stride kPartialPad);
// if z != null also z[i*b + t] = s[i] * new value.
hipError_t launch_apply_rinv(double* basis, int64_t n, int64_t ld, int col0, int b, const double* rinv, double* z,
                             const double* s, hipStream_t st);

// Fused variant used inside the block step (same arithmetic as the separate kernels):
//   update_gram: basis[:, ccol0 : ccol0+b] -= basis[:, acol0 : acol0+kdim] * bmat (bmat kdim x b, row stride
//                kPartialPad) and
//                gpart[p] (b x b, row stride kPartialPad, p < plan_update_gram(n)) = partial Gram matrices of the
//                updated block, to be summed with launch_reduce_partials(gpart, npart, b, b, ...).
int plan_update_gram(int64_t n);
// overwrite = 1: the block is replaced by the product instead of having it subtracted (W <- W R^-1 with
// acol0 = ccol0, kdim = b, bmat = R^-1); overwrite = 2: the product is subtracted for the Gram matrix only, the block
// in memory stays as it is
hipError_t launch_update_gram(double* basis, int64_t n, int64_t ld, int acol0, int kdim, const double* bmat, int b,
                              int ccol0, int overwrite, double* gpart, hipStream_t st, const int* skip = nullptr);
// ---- Chebyshev filter with the iterates resident in LDS (resident.hip) -------------------------------
// A work item is a diagonal block (or a 16-column slice of it) worked on by lane groups of cl = 4 lanes (32 columns)
// or cl = 2 lanes (16 columns).  Its rows are cut into chunks of 8 cl entries; `extra` = chunks beyond the first,
// summed over its rows.  LDS bytes of an item, and the largest number of chunks (rows + extra) one may have:
size_t resident_item_lds_bytes(int nrows, int cl, int extra);
int resident_max_chunks(int cl);
// Diagonal blocks of a CSR matrix with a symmetric pattern: starts[0 .. *count) = the rows p (ascending) such that no
// row before p has an entry in column p or beyond; starts has room for n entries, count is a device int32.
// work: device scratch of diagonal_blocks_workspace(n) bytes.  n <= INT32_MAX.
size_t diagonal_blocks_workspace(int64_t n);
hipError_t diagonal_blocks(const int64_t* rowptr, const int32_t* col, int64_t n, void* work, size_t work_bytes,
                           int32_t* starts, int32_t* count, hipStream_t st);
// extra[2 t], extra[2 t + 1] (device int32) = extra chunks of block t for chunks of 32 and of 16 entries
hipError_t launch_block_extra_chunks(const int64_t* rowptr, const int32_t* starts, int nblk, int64_t n, int32_t* extra,
                                     hipStream_t st);
// y (n x b, leading dimension ldy >= b) = the recurrence applied to x (packed n x b): u_0 = x, u_1 = alpha_first (A u_0 - shift u_0),
// u_{i+1} = alpha_rest (A u_i - shift u_i) - u_{i-1}; y = u_d.  A = the CSR matrix, whose rows [row0, row0 + nrows) of
// every item form a diagonal block.  items: device int32[4 * nitems] = (row0, nrows, col0, cl | extra << 4) per
// workgroup, covering columns [col0, col0 + 8 cl); every (block, column) pair must be covered exactly once, extra must
// be the block's extra-chunk count for chunks of 8 cl entries and nrows + extra <= resident_max_chunks(cl).
// lds_bytes = the largest resident_item_lds_bytes over the items.  y must not alias x.
// A sliced item (cl = 1; the word's upper bits carry the item's first slice, not a chunk count) covers 8 columns of a
// block of up to 65,535 rows and reads its entries from the sliced copy (scol, sval, slice_base, slice_len; null when
// no item is sliced).
// d32 (0 <= d32 < d): the first d32 steps of the items with cl = 2 or 4 run in single precision (iterates and entries
// rounded to float), the rest in double; sliced items take all steps in double.  0 gives the recurrence in double.
// use_rnd != 0: x is not read; the operand is the random block of key rnd_key (random_block_key), entry by entry as
// launch_random_block would have written it into a packed n x b buffer.
hipError_t launch_cheb_resident(const int64_t* rowptr, const int32_t* col, const double* val, const double* x, double* y,
                                int64_t ldy, int b, int d, double alpha_first, double alpha_rest, double shift, const int32_t* items,
                                int nitems, size_t lds_bytes, const uint16_t* scol, const double* sval,
                                const int64_t* slice_base, const int32_t* slice_len, hipStream_t st, int d32 = 0,
                                uint64_t rnd_key = 0, int use_rnd = 0);
// key of random block number `stream_id` under `seed`: entry i * b + t of the block launch_random_block writes is
// 2 u - 1 with u the top 53 bits of mix(key + i * b + t)
uint64_t random_block_key(uint64_t seed, uint64_t stream_id);
// Sliced copy of diagonal blocks for the sliced form.  A slice is up to resident_slice_rows() consecutive rows of one
// block: slice_row0 / slice_rows (device int32[nslices]) name its rows, slice_blk0 / slice_blk_rows its block.
// sliced_copy_layout fills slice_len (longest row), slice_entries (int64[nslices + 1]: entries the slice takes in the
// copy, padding included; last slot 0) and slice_base (int64[nslices + 1]: exclusive prefix sums; the last one is the
// size of the copy).  sliced_copy_fill writes the copy: scol / sval with room for slice_base[nslices] +
// sliced_copy_tail_entries() entries (the kernel's requests run that far past the last slice; initialise the tail).
int resident_slice_rows();
int64_t sliced_copy_tail_entries();
size_t resident_sliced_lds_bytes(int nrows);
size_t sliced_scan_workspace(int nslices);
hipError_t sliced_copy_layout(const int64_t* rowptr, const int32_t* slice_row0, const int32_t* slice_rows, int nslices,
                              int32_t* slice_len, int64_t* slice_entries, int64_t* slice_base, void* work,
                              size_t work_bytes, hipStream_t st);
hipError_t sliced_copy_fill(const int64_t* rowptr, const int32_t* col, const double* val, const int32_t* slice_row0,
                            const int32_t* slice_rows, const int32_t* slice_blk0, const int32_t* slice_blk_rows,
                            int nslices, const int64_t* slice_base, const int64_t* slice_entries, uint16_t* scol,
                            double* sval, hipStream_t st);

// ---- connected components and locality reordering (setup) --------------------------------------
// Renumbering from the component labels (label[i] = smallest node index of i's component), on the device:
//   old_of_new[p] = original index of new row p (components contiguous, ordered by their smallest node; inside a
//   component by three levels of neighbourhood min-hash, ties in original order), new_of_old = its inverse,
//   rowptr_new (n+1) = row pointers of the permuted matrix, comp_of_new[p] = component index of new row p.
// work: device scratch of order_by_component_workspace(n) bytes.  All outputs are device arrays; n <= INT32_MAX.
size_t order_by_component_workspace(int64_t n);
// by_length != 0: on a graph with hubs (longest row > 3 average rows) the rows of a component are ordered by decreasing
// length first (for the wide sparse products), then by the min-hash levels.  big_rows > 0: the components with more
// nodes than that come after all the others (in the order of their smallest node among themselves).
hipError_t order_by_component(const int64_t* rowptr, const int32_t* col, const int32_t* label, int64_t n, int by_length,
                              int big_rows, void* work,
                              size_t work_bytes, int32_t* old_of_new, int32_t* new_of_old, int64_t* rowptr_new,
                              int32_t* comp_of_new, hipStream_t st);
// list[0 .. *count) = the rows with more than kLongRow entries, ascending; list has room for n entries; count: device
// int32.  work: device scratch of long_row_list_workspace(n) bytes.
size_t long_row_list_workspace(int64_t n);
hipError_t long_row_list(const int64_t* rowptr, int64_t n, void* work, size_t work_bytes, int32_t* list, int32_t* count,
                         hipStream_t st);
// label[i] = i
hipError_t launch_iota(int32_t* label, int64_t n, hipStream_t st);
// one round of minimum-label propagation with pointer jumping; *changed = 1 if a label moved
hipError_t launch_cc_round(const int64_t* rowptr, const int32_t* col, const double* val, int32_t* label, int64_t n,
                           int* changed, hipStream_t st);
// permuted CSR: row p = input row old_of_new[p], column c renamed new_of_old[c]; rowptr_new precomputed
hipError_t launch_permute_csr(const int64_t* rowptr, const int32_t* col, const double* val, const int32_t* old_of_new,
                              const int32_t* new_of_old, const int64_t* rowptr_new, int32_t* col_new, double* val_new,
                              int64_t n, hipStream_t st);
// basis[i, col0 + t] = comp[i] == t ? coef[i] : 0  for t < ncols (closed-form null vectors of the components)
hipError_t launch_nullspace_fill(double* basis, int64_t n, int64_t ld, int col0, int ncols, const int32_t* comp,
                                 const double* coef, hipStream_t st);

// ---- misc ----------------------------------------------------------------------------------
// dst[i*ldd + dcol0 + t] -= src[i*lds + scol0 + t], t < w (regions must not overlap)
hipError_t launch_sub_cols(const double* src, int64_t lds, int scol0, double* dst, int64_t ldd, int dcol0, int w,
                           int64_t n, hipStream_t st);
// basis[i*ld + col] = v[rowmap ? rowmap[i] : i]
hipError_t launch_set_column(double* basis, int64_t n, int64_t ld, int col, const double* v, const int32_t* rowmap,
                             hipStream_t st);
// basis[i, col0 + t] = uniform(-1, 1) from a counter-based hash of (seed, stream_id, i, t)
hipError_t launch_random_block(double* basis, int64_t n, int64_t ld, int col0, int b, uint64_t seed,
                               uint64_t stream_id, hipStream_t st);
// dst[i*ldd + dcol0 + t] = src[i*lds + scol0 + t], t < w (regions must not overlap)
// out[pos[c]*n + o] = basis[r(o)*ld + c] for c < ncols with pos[c] >= 0 (pos: device int32[ncols], the output column
// of basis column c or -1; r(o) = inv[o], the internal row of original row o, if inv is given, else o)
hipError_t launch_gather_cols_colmajor(const double* basis, int64_t n, int64_t ld, const int32_t* pos, int ncols,
                                       double* out, const int32_t* inv, hipStream_t st);
// The solver's own operator copy for wide blocks (b = 8, 16, 32) holds S_ij = s_i W_ij s_j multiplied out:
// val_out[e] = s_i * val[e] * s_j (val_out may be val).
hipError_t launch_scale_values(const int64_t* rowptr, const int32_t* col, const double* val, const double* s,
                               double* val_out, int64_t n, hipStream_t st);
// y = A x with the values as stored (the scaled copy); x packed n x b (b = 8, 16, 32; 16-byte aligned), y row-major
// with leading dimension ldy.
// longrows (may be null): device list of the nlong rows with more than kLongRow entries, ascending (long_row_list);
// those rows are then computed by a workgroup each instead of a lane group.
hipError_t launch_spmm_vals(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, const double* x,
                            int b, double* y, int64_t ldy, double avg_deg, const int32_t* longrows, int nlong,
                            hipStream_t st);
// One Chebyshev recurrence step on packed blocks:  unext = alpha * (A ucur - shift * ucur) - beta * uprev
// (uprev is not read when beta == 0; unext must not be ucur).  row_begin > 0: only the rows [row_begin, n) are computed
// and written (the rows before it belong to a caller that computes them another way).
hipError_t launch_spmm_vals_cheb(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n,
                                 const double* ucur, int b, const double* uprev, double* unext, double alpha,
                                 double shift, double beta, double avg_deg, const int32_t* longrows, int nlong,
                                 hipStream_t st, int64_t row_begin = 0);
// out[t*n + o] *= s[r(o)], t < k (column-major vectors in the caller's numbering; s in the internal numbering)
hipError_t launch_scale_rows_colmajor(double* out, int64_t n, int k, const double* s, const int32_t* inv, hipStream_t st);
// every row of the n x k column-major matrix scaled to unit 2-norm (zero rows stay zero)
hipError_t launch_normalize_rows_colmajor(double* out, int64_t n, int k, hipStream_t st);
// ynext = alpha (w - shift ycur) - beta yprev and znext = s o ynext on packed n x b blocks (Chebyshev recurrence step)
hipError_t launch_cheb_combine(const double* w, const double* ycur, const double* yprev, const double* s, double alpha,
                               double shift, double beta, double* ynext, double* znext, int64_t n, int b,
                               hipStream_t st);
hipError_t launch_copy_cols(const double* src, int64_t lds, int scol0, double* dst, int64_t ldd, int dcol0, int w,
                            int64_t n, hipStream_t st);

// ---- k-means on the embedding (Section IV-C, Algorithms 4-5; kmeans.hip) ------------------------
// x (n x ldx row-major, zero padded beyond d) from the caller's points (column-major v[t*ldv + i] or row-major)
hipError_t launch_points_to_rowmajor(const double* v, int64_t ldv, int colmajor, int64_t n, int d, double* x, int64_t ldx,
                                     hipStream_t st);
// ct (dpad x ldc row-major) = transpose of the k x ldx centre array, cnorm[j] = |c_j|^2
hipError_t launch_centroid_operand(const double* c, int64_t ldx, int k, int d, int dpad, double* ct, int64_t ldc,
                                   double* cnorm, hipStream_t st);
// label[i] = arg-min_j cnorm[j] - 2 s[i, j] (first on ties); *changes += number of labels that changed
hipError_t launch_argmin(const double* s, int64_t lds, int64_t n, int k, const double* cnorm, int32_t* label,
                         int* changes, hipStream_t st);
hipError_t launch_fill_int32(int32_t* a, int64_t n, int32_t value, int use_iota, hipStream_t st);
// centres = means of their points (sort by label, fixed summation order); empty clusters keep their centre.
// work: kmeans_update_workspace(n) bytes; start: device int32[k+1] (first sorted position of every cluster)
size_t kmeans_update_workspace(int64_t n);
hipError_t launch_centroid_update(const double* x, int64_t ldx, int d, int64_t n, const int32_t* label, int k, void* work,
                                  size_t work_bytes, int32_t* start, double* c, hipStream_t st);
// Algorithm 5 with the uniform numbers u[0..k-1] supplied by the host; chosen: device int32[k]
size_t kmeans_seed_workspace(int64_t n);
hipError_t launch_kmeanspp(const double* x, int64_t ldx, int d, int64_t n, int k, const double* u, void* work,
                           size_t work_bytes, int32_t* chosen, hipStream_t st);
hipError_t launch_gather_rows(const double* x, int64_t ldx, const int32_t* index, int k, double* c, hipStream_t st);
// part[p], p < kmeans_objective_parts(): partial sums of |x_i - c_label(i)|^2 (add them in order on the host)
int kmeans_objective_parts();
hipError_t launch_objective(const double* x, int64_t ldx, int d, int64_t n, const int32_t* label, const double* c,
                            double* part, hipStream_t st);
hipError_t launch_copy_rows(const double* src, int64_t lds, double* dst, int64_t ldd, int rows, int cols, hipStream_t st);

// ---- similarity graph (Section IV-A, Algorithm 1; Algorithm 2 step 4; similarity.hip) ----------------------------
// mean[i] = row mean (0 if centre == 0), norm[i] = 2-norm of the row minus that mean; x row-major n x ldx
hipError_t launch_row_stats(const double* x, int64_t ldx, int64_t n, int d, int centre, double* mean, double* norm,
                            hipStream_t st);
// measure 0 cross correlation, 1 cosine (both with mean/norm from launch_row_stats), 2 exp(-|xu-xv|^2 / (2 sigma^2));
// *bad |= 1 and val[e] = NaN for an edge with an index outside [0, n)
hipError_t launch_edge_similarity(const double* x, int64_t ldx, int d, const int32_t* eu, const int32_t* ev,
                                  int64_t nedges, int measure, double sigma, const double* mean, const double* norm,
                                  int64_t n, int* bad, double* val, hipStream_t st);
// ---- k-nearest-neighbour graph (Section III-A; knn.hip) -------------------------------------------------------
// Exact Euclidean k nearest neighbours of every row of x (n x d, leading dimension ldx) other than the row itself:
// idx_out[i*k + a] / dist_out[i*k + a] = index / distance of the a-th nearest, nearest first, equal distances by
// index.  xp: device scratch of n * (knn_padded_dim(d) + 1) doubles.  2 <= n <= INT32_MAX, 1 <= k <= n - 1, and
// knn_search_lds_bytes(d, k) must not exceed the LDS a workgroup may have (else hipErrorInvalidValue).
int knn_padded_dim(int d);
size_t knn_search_lds_bytes(int d, int k);
hipError_t launch_knn_search(const double* x, int64_t ldx, int64_t n, int d, int k, double* xp, int32_t* idx_out,
                             double* dist_out, hipStream_t st);
// The undirected edges {i, j} (j in i's list or i in j's) once each as eu < ev, in row order of the emitting list;
// val = the listed distance, or exp(-dist^2 / (2 sigma^2)) if sigma > 0.  eu, ev, val have room for n * k entries;
// last_two (device int32[2]) receives two numbers whose sum is the pair count.  work: knn_pairs_workspace(n) bytes.
size_t knn_pairs_workspace(int64_t n);
hipError_t launch_knn_union_pairs(const int32_t* idx, const double* dist, int64_t n, int k, double sigma, void* work,
                                  size_t work_bytes, int32_t* eu, int32_t* ev, double* val, int32_t* last_two,
                                  hipStream_t st);
size_t coo_to_csr_workspace(int64_t total);
hipError_t coo_to_csr(const int32_t* row, const int32_t* col, const double* val, int64_t nnz_in, int64_t n,
                      int symmetrize, void* work, size_t work_bytes, int64_t* rowptr_out, int32_t* col_out,
                      double* val_out, int* bad, hipStream_t st);

// Measurement aid: `workgroups` workgroups of four waves, each wave issuing iters * 8 fp64 matrix instructions and
// nothing else; shape 16: 16x16x4 (2,048 flops each), shape 4: 4x4x4 (512 flops each); sink: device, workgroups * 256
// doubles.
hipError_t launch_mfma_rate(double* sink, int shape, int workgroups, int iters, hipStream_t st);

}  // namespace sceig
