// HIP kernels for gfx950 (CDNA4, wave64).  See kernels.h for the contracts.
//
// fp64 MFMA operand layout used below (v_mfma_f64_16x16x4_f64, one wave):
//   A (16 x 4):  lane l holds A[l % 16][l / 16]
//   B (4 x 16):  lane l holds B[l / 16][l % 16]
//   D (16 x 16): lane l, register r (0..3) holds D[4*r + l / 16][l % 16]
#include "kernels.h"

namespace sceig {

typedef double d4 __attribute__((ext_vector_type(4)));

#define MFMA_F64(a, b, c) __builtin_amdgcn_mfma_f64_16x16x4f64((a), (b), (c), 0, 0, 0)

namespace {

constexpr int kThreads = 256;

__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// --------------------------------------------------------------------------------------------
// setup
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void validate_rowptr_kernel(const int64_t* __restrict__ rowptr, int64_t n,
                                                                   int64_t nnz, int* __restrict__ flag) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n) return;
  const int64_t a = rowptr[i], b = rowptr[i + 1];
  bool bad = a > b || a < 0 || b > nnz;
  if (i == 0 && a != 0) bad = true;
  if (bad) atomicOr(flag, 1);
}

__global__ __launch_bounds__(kThreads) void validate_col_kernel(const int32_t* __restrict__ col, int64_t nnz, int64_t n,
                                                                int* __restrict__ flag) {
  int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  bool bad = false;
  for (; e < nnz; e += stride) {
    const int32_t c = col[e];
    bad |= (c < 0) | ((int64_t)c >= n);
  }
  if (bad) atomicOr(flag, 2);
}

// Symmetry and sign of the weights, one wave per row.  For every entry (i, j) the weights of row i listed under
// column j must add up to the weights of row j listed under column i (rows may be unsorted and may list a column
// more than once, so both sides are summed in storage order); equality is required up to four units in the last
// place of the larger side, the most that two different summation orders of a handful of duplicates can differ by.
// flag |= 8 if some pair differs, |= 16 if a weight is negative or not finite.
__global__ __launch_bounds__(kThreads) void validate_symmetry_kernel(const int64_t* __restrict__ rowptr,
                                                                     const int32_t* __restrict__ col,
                                                                     const double* __restrict__ val, int64_t n,
                                                                     int* __restrict__ flag) {
  const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (i >= n) return;
  const int64_t a0 = rowptr[i], a1 = rowptr[i + 1];
  int bad = 0;
  for (int64_t e = a0 + lane; e < a1; e += 64) {
    const int32_t j = col[e];
    const double w = val[e];
    if (!(w >= 0.0) || isinf(w)) bad |= 16;
    double mine = 0.0, theirs = 0.0;
    for (int64_t f = a0; f < a1; ++f) mine += col[f] == j ? val[f] : 0.0;
    const int64_t b0 = rowptr[j], b1 = rowptr[j + 1];
    for (int64_t f = b0; f < b1; ++f) theirs += (int64_t)col[f] == i ? val[f] : 0.0;
    const double big = fmax(fabs(mine), fabs(theirs));
    if (!(fabs(mine - theirs) <= 8.9e-16 * big)) bad |= 8;
  }
  if (bad) atomicOr(flag, bad);
}

// 16 lanes per row
__global__ __launch_bounds__(kThreads) void degree_kernel(const int64_t* __restrict__ rowptr,
                                                          const double* __restrict__ val, int64_t n,
                                                          double* __restrict__ d, double* __restrict__ s,
                                                          int* __restrict__ flag) {
  const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 4;
  const int lane = threadIdx.x & 15;
  if (row >= n) return;  // uniform over the 16-lane group
  const int64_t e1 = rowptr[row + 1];
  double acc = 0.0;
  for (int64_t e = rowptr[row] + lane; e < e1; e += 16) acc += val[e];
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 16);
  if (lane == 0) {
    if (d) d[row] = acc;
    s[row] = 1.0 / sqrt(acc);
    if (!(acc > 0.0) || isinf(acc)) atomicOr(flag, 4);
  }
}

// --------------------------------------------------------------------------------------------
// sparse product
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void pack_scaled_kernel(const double* __restrict__ x, int64_t ldx,
                                                               const double* __restrict__ s, int64_t n, int b,
                                                               double* __restrict__ z) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * b) return;
  const int64_t i = idx / b;
  const int t = (int)(idx - i * b);
  z[idx] = s ? s[i] * x[i * ldx + t] : x[i * ldx + t];
}

// Workgroups are handed to the 8 XCDs (each with an L2 of its own) round-robin by their linear index.  The sparse
// products gather rows of z that lie near the rows they compute (the solver numbers every connected component
// contiguously), so each XCD should own one contiguous eighth of the row tiles instead of every eighth tile: then an
// L2 holds an eighth of z rather than all of it.  The grid must be a multiple of kXcds; tiles past the end are idle.
constexpr int kXcds = 8;
__device__ __forceinline__ int64_t xcd_tile() {
  return (int64_t)(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds;
}
static inline unsigned xcd_grid(int64_t tiles) { return (unsigned)(ceil_div64(tiles, kXcds) * kXcds); }

// L lanes per row, B = 8, 16, 32 columns.  The L lanes load L consecutive (col, val) pairs of the row at once.  A
// lane carries TWO adjacent columns of the block, so CL = B/2 lanes cover one entry with 16-byte gathers, and the
// NS = L/CL sub-groups split the batch round-robin (entry r*NS + g goes to sub-group g in round r).  A row of up to
// L entries is one load -> gather -> sum chain; long rows (hubs of the kNN graph) take deg/L trips.  The sub-group
// sums are combined in a fixed order by a shuffle tree.
//
// MODE 0: y = s o (W z), z = s o x packed by the caller (the operator applied from W and the scaling vector).
// MODE 1: y = A z with the values as they are (the solver's copy holds S_ij = s_i W_ij s_j already multiplied out,
//         as Algorithm 2's scaling step does), z = x packed.
// MODE 2: one step of the Chebyshev recurrence on packed blocks with such values:
//         y = alpha * (A z - shift * z) - beta * uprev   (uprev is not read when beta == 0; y packed, ldy = B).
// Long rows.  A kNN graph of high-dimensional points has hubs: on the 100,000-node workload the median row has 24
// entries, one in a hundred more than 124 and the longest 432, and a row that one lane group walks batch after batch
// is a serial chain of dependent loads that the whole launch ends up waiting for.  When the caller passes the list
// of rows longer than kLongRow entries, the row tiles skip them and extra workgroups at the end of the grid take one
// long row each: the G lane groups of the workgroup take its batches round-robin and their partial sums are added in
// group order (fixed, so results stay reproducible).  Measured on that workload at B = 16: 36.4 -> 30.7 us.
template <int B, int L, int MODE>
__global__ __launch_bounds__(kThreads) void spmm_cols_kernel(const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col,
                                                             const double* __restrict__ val,
                                                             const double* __restrict__ s,
                                                             const double* __restrict__ z, double* __restrict__ y,
                                                             int64_t ldy, int64_t n, int vec_store,
                                                             const double* __restrict__ uprev, double alpha,
                                                             double shift, double beta, int64_t ntiles,
                                                             const int32_t* __restrict__ longrows, int nlong,
                                                             int64_t row_begin) {
  constexpr int G = kThreads / L;  // lane groups per workgroup
  constexpr int CL = B / 2;        // lanes per entry
  static_assert(L % CL == 0, "batch must split evenly");
  constexpr int NS = L / CL;        // sub-groups of a row
  __shared__ double part[G][B];
  const int lane = threadIdx.x % L;
  const int tl = lane % CL;
  const int sg = lane / CL;         // this lane's sub-group
  const int gi = threadIdx.x / L;
  const bool main_part = (int64_t)blockIdx.x < ntiles;
  int64_t row, e_first, e_step;
  if (main_part) {
    // row tiles, handed to the XCDs in contiguous eighths (ntiles is a multiple of kXcds)
    const int64_t tile = (int64_t)(blockIdx.x % kXcds) * (ntiles / kXcds) + blockIdx.x / kXcds;
    row = row_begin + tile * G + gi;  // rows before row_begin are somebody else's (see launch_spmm_vals_cheb)
    if (row >= n) return;  // uniform over the L-lane group; this part has no workgroup barrier
    e_first = 0;
    e_step = L;
  } else {
    const int64_t bl = (int64_t)blockIdx.x - ntiles;
    const int64_t per = ((int64_t)nlong + kXcds - 1) / kXcds;
    const int64_t li = (bl % kXcds) * per + bl / kXcds;
    if (li >= nlong) return;  // uniform over the workgroup
    row = longrows[li];
    if (row < row_begin) return;  // uniform over the workgroup
    e_first = (int64_t)gi * L;
    e_step = (int64_t)G * L;
  }
  const int64_t e0 = rowptr[row], e1 = rowptr[row + 1];
  if (main_part && longrows && e1 - e0 > kLongRow) return;  // done by a workgroup of its own
  double acc0 = 0.0, acc1 = 0.0;
  const double2* __restrict__ z2 = reinterpret_cast<const double2*>(z);
  double2 cur = {0.0, 0.0}, pv = {0.0, 0.0};
  if constexpr (MODE == 2) {
    if (lane < CL && (main_part || gi == 0)) {  // the recurrence's own-row operands, requested ahead of the gathers
      cur = z2[row * CL + tl];
      if (beta != 0.0) pv = reinterpret_cast<const double2*>(uprev)[row * CL + tl];
    }
  }
  for (int64_t e = e0 + e_first; e < e1; e += e_step) {
    // Lanes past the end of the row load the row's last entry again and take the value 0: their products vanish.
    // The loads are unconditional on purpose: defaults written to the same registers before a conditional load make
    // the compiler wait for every load still in flight (the recurrence's own-row operands, requested above) before
    // this one is even issued.
    const int64_t el = e + lane < e1 ? e + lane : e1 - 1;
    const int32_t c = col[el];
    const double av = val[el];
    const double a = e + lane < e1 ? av : 0.0;
    // The batch's entries go round-robin to the NS sub-groups (entry r*NS + g to sub-group g in round r), so a batch
    // of cnt entries costs ceil(cnt / NS) gather instructions: a row of 24 entries takes 6 rounds at B = 16, the
    // one-entry tail of a row of 33 takes 1.
    const int cnt = (e1 - e) < L ? (int)(e1 - e) : L;  // uniform over the row's lanes
    const int rounds = (cnt + NS - 1) / NS;
    int r = 0;
#define SC_GATHER_ROUNDS(K)                                  \
  {                                                          \
    double2 zv[K];                                           \
    _Pragma("unroll") for (int u = 0; u < K; ++u) {          \
      const int32_t cu = __shfl(c, (r + u) * NS + sg, L);    \
      zv[u] = z2[(int64_t)cu * CL + tl];                     \
    }                                                        \
    _Pragma("unroll") for (int u = 0; u < K; ++u) {          \
      const double au = __shfl(a, (r + u) * NS + sg, L);     \
      acc0 += au * zv[u].x;                                  \
      acc1 += au * zv[u].y;                                  \
    }                                                        \
    r += K;                                                  \
  }
    while (rounds - r >= 4) SC_GATHER_ROUNDS(4)
    if (rounds - r >= 2) SC_GATHER_ROUNDS(2)
    if (rounds - r >= 1) SC_GATHER_ROUNDS(1)
#undef SC_GATHER_ROUNDS
  }
#pragma unroll
  for (int o = L / 2; o >= CL; o >>= 1) {
    acc0 += __shfl_xor(acc0, o, L);
    acc1 += __shfl_xor(acc1, o, L);
  }
  if (!main_part) {  // the G groups' partial sums of the long row, added in group order by group 0
    if (lane < CL) {
      part[gi][2 * tl] = acc0;
      part[gi][2 * tl + 1] = acc1;
    }
    __syncthreads();
    if (gi != 0) return;
    acc0 = 0.0;
    acc1 = 0.0;
    if (lane < CL) {
#pragma unroll
      for (int q = 0; q < G; ++q) {
        acc0 += part[q][2 * tl];
        acc1 += part[q][2 * tl + 1];
      }
    }
  }
  if (lane < CL) {
    if constexpr (MODE == 2) {
      double2 out;
      out.x = alpha * (acc0 - shift * cur.x) - beta * pv.x;
      out.y = alpha * (acc1 - shift * cur.y) - beta * pv.y;
      reinterpret_cast<double2*>(y)[row * CL + tl] = out;
    } else {
      const double sr = MODE == 0 ? s[row] : 1.0;
      if (vec_store) {  // one 16-byte store (y + row * ldy is 16-byte aligned)
        double2 out;
        out.x = sr * acc0;
        out.y = sr * acc1;
        *reinterpret_cast<double2*>(y + row * ldy + 2 * tl) = out;
      } else {
        y[row * ldy + 2 * tl] = sr * acc0;
        y[row * ldy + 2 * tl + 1] = sr * acc1;
      }
    }
  }
}

// val_out[e] = s_i * val[e] * s_j for entry e = (i, j): the scaled copy of the operator.  The same rounding for
// (i, j) and (j, i), so the copy is exactly symmetric when W is.  val_out may be val.
__global__ __launch_bounds__(kThreads) void scale_values_kernel(const int64_t* __restrict__ rowptr,
                                                                const int32_t* __restrict__ col, const double* val,
                                                                const double* __restrict__ s, double* val_out,
                                                                int64_t n) {
  constexpr int L = 16;  // lanes per row
  const int lane = threadIdx.x % L;
  const int64_t row = (int64_t)blockIdx.x * (kThreads / L) + threadIdx.x / L;
  if (row >= n) return;
  const double si = s[row];
  const int64_t e1 = rowptr[row + 1];
  for (int64_t e = rowptr[row] + lane; e < e1; e += L) {
    const int32_t c = col[e];
    const double sj = s[c];
    const double ss = (int64_t)c < row ? sj * si : si * sj;
    val_out[e] = val[e] * ss;
  }
}

// L lanes per row, each lane walks the entries of the row with stride L and keeps B accumulators
// (B = 1, 2, 4); the L partial sums are combined by a shuffle tree.
template <int B, int L>
__global__ __launch_bounds__(kThreads) void spmm_nz_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const double* __restrict__ val,
                                                           const double* __restrict__ s,
                                                           const double* __restrict__ z, double* __restrict__ y,
                                                           int64_t ldy, int64_t n) {
  constexpr int G = kThreads / L;
  const int t = threadIdx.x % L;
  const int64_t row = (int64_t)blockIdx.x * G + threadIdx.x / L;
  if (row >= n) return;  // uniform over the L-lane group
  const int64_t e1 = rowptr[row + 1];
  double acc[B];
#pragma unroll
  for (int q = 0; q < B; ++q) acc[q] = 0.0;
  for (int64_t e = rowptr[row] + t; e < e1; e += 2 * L) {
    const bool ok1 = e + L < e1;
    const int64_t c0 = col[e], c1 = ok1 ? col[e + L] : 0;
    const double a0 = val[e], a1 = ok1 ? val[e + L] : 0.0;
#pragma unroll
    for (int q = 0; q < B; ++q) acc[q] += a0 * z[c0 * B + q] + a1 * z[c1 * B + q];
  }
#pragma unroll
  for (int o = L / 2; o > 0; o >>= 1) {
#pragma unroll
    for (int q = 0; q < B; ++q) acc[q] += __shfl_xor(acc[q], o, L);
  }
  if (t == 0) {
    const double sr = s ? s[row] : 1.0;
#pragma unroll
    for (int q = 0; q < B; ++q) y[row * ldy + q] = sr * acc[q];
  }
}

// Row-block streaming product for narrow blocks (B = 1, 2, 4): a workgroup owns RB consecutive rows, streams their
// entries fully coalesced (eight independent entry loads and gathers per thread in flight), parks the products
// val * z[col] in LDS and then sums every row from LDS with 256/RB lanes.  No row is split between workgroups
// and the order of every sum is fixed by the row's position, so results are reproducible.
template <int B, int RB>
__global__ __launch_bounds__(kThreads) void spmm_stream_kernel(const int64_t* __restrict__ rowptr,
                                                               const int32_t* __restrict__ col,
                                                               const double* __restrict__ val,
                                                               const double* __restrict__ s,
                                                               const double* __restrict__ z, double* __restrict__ y,
                                                               int64_t ldy, int64_t n) {
  constexpr int CH = 2048 / B;       // entries per LDS chunk
  constexpr int LR = kThreads / RB;  // lanes per row in the summation
  __shared__ double prod[CH * B];
  __shared__ int64_t rp[RB + 1];
  const int64_t r0 = xcd_tile() * RB;
  if (r0 >= n) return;  // idle tile of the rounded-up grid (uniform over the workgroup)
  const int nrows = (int)((n - r0) < RB ? (n - r0) : RB);
  if (threadIdx.x <= nrows) rp[threadIdx.x] = rowptr[r0 + threadIdx.x];
  __syncthreads();
  const int64_t e_begin = rp[0], e_end = rp[nrows];
  const int rl = threadIdx.x / LR, lane = threadIdx.x % LR;
  double acc[B];
#pragma unroll
  for (int q = 0; q < B; ++q) acc[q] = 0.0;
  for (int64_t c0 = e_begin; c0 < e_end; c0 += CH) {
    const int64_t c1 = (c0 + CH) < e_end ? (c0 + CH) : e_end;
    for (int64_t base = c0 + threadIdx.x; base < c1; base += 4 * kThreads) {
      int32_t c[4];
      double a[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool ok = base + u * kThreads < c1;
        c[u] = ok ? col[base + u * kThreads] : 0;
        a[u] = ok ? val[base + u * kThreads] : 0.0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (base + u * kThreads < c1) {
#pragma unroll
          for (int q = 0; q < B; ++q)
            prod[(base + u * kThreads - c0) * B + q] = a[u] * z[(int64_t)c[u] * B + q];
        }
      }
    }
    __syncthreads();
    if (rl < nrows) {
      int64_t lo = rp[rl] > c0 ? rp[rl] : c0;
      const int64_t hi = rp[rl + 1] < c1 ? rp[rl + 1] : c1;
      for (int64_t e = lo + lane; e < hi; e += LR) {
#pragma unroll
        for (int q = 0; q < B; ++q) acc[q] += prod[(e - c0) * B + q];
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int o = LR / 2; o > 0; o >>= 1) {
#pragma unroll
    for (int q = 0; q < B; ++q) acc[q] += __shfl_xor(acc[q], o, LR);
  }
  if (lane == 0 && rl < nrows) {
    const double sr = s ? s[r0 + rl] : 1.0;
#pragma unroll
    for (int q = 0; q < B; ++q) y[(r0 + rl) * ldy + q] = sr * acc[q];
  }
}

// Single-vector product, one wave per tile of RW consecutive rows.  The wave requests the tile's whole (col, val)
// stream at once - entry u*64 + lane in lane's registers, so every load instruction covers 64 consecutive entries -,
// then the gathers z[col], parks the products in its own LDS strip and sums every row from there with 64/RW lanes.
// No workgroup barrier: the four waves of a workgroup never wait for each other, and because every wave is short
// lived the tiles in flight form one window that moves through the matrix in memory order.  All index arithmetic
// inside the tile is 32-bit on a wave-uniform base.  Loads past the tile's end are clamped to its last entry (their
// products are never summed) instead of being predicated.  Tiles with more than U*64 entries take further chunks on
// demand.  The order of every row sum is fixed by the row's position in its tile.
__device__ __forceinline__ int64_t readlane64(int64_t v, int l) {
  const int lo = __builtin_amdgcn_readlane((int)v, l);
  const int hi = __builtin_amdgcn_readlane((int)(v >> 32), l);
  return ((int64_t)hi << 32) | (uint32_t)lo;
}

template <int RW, int U>
__global__ __launch_bounds__(kThreads) void spmv_tile_kernel(const int64_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ col,
                                                             const double* __restrict__ val,
                                                             const double* __restrict__ s,
                                                             const double* __restrict__ z, double* __restrict__ y,
                                                             int64_t ldy, int64_t n, int64_t ntiles,
                                                             double* __restrict__ zout) {
  constexpr int LR = 64 / RW;  // lanes per row in the summation
  constexpr int CH = U * 64;   // entries per chunk
  __shared__ double prod_all[kThreads / 64][CH];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  double* prod = prod_all[wave];
  const int64_t tile = (int64_t)blockIdx.x * (kThreads / 64) + wave;
  if (tile >= ntiles) return;  // wave-uniform; there is no workgroup barrier below
  const int g = lane / LR, sl = lane % LR;
  const int64_t row0 = tile * RW;
  int64_t r = row0 + lane;
  r = r < n ? r : n;  // rows past the end are empty: their pointers equal rowptr[n]
  const int64_t rpv = lane <= RW ? rowptr[r] : 0;
  const int64_t e0 = readlane64(rpv, 0);
  const int len = (int)(readlane64(rpv, RW) - e0);
  const bool mine = sl == 0 && row0 + g < n;
  // the row's scaling factor, requested now by the lane that writes the row and needed only at the very end
  // (s == null: the values are S already)
  const double sg = (mine && s) ? s[row0 + g] : 1.0;
  if (len <= 0) {
    if (mine) {
      y[(row0 + g) * ldy] = 0.0;
      if (zout) zout[row0 + g] = 0.0;
    }
    return;
  }
  const int32_t* cp = col + e0;
  const double* vp = val + e0;
  int32_t c[U];
  double a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int idx = u * 64 + lane;
    idx = idx < len ? idx : len - 1;
    c[u] = cp[idx];
    a[u] = vp[idx];
  }
  const int rel = (int)(rpv - e0);
  const int rlo = __shfl(rel, g), rhi = __shfl(rel, g + 1);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const double zz = *reinterpret_cast<const double*>(reinterpret_cast<const char*>(z) + ((uint64_t)(uint32_t)c[u] << 3));
    prod[u * 64 + lane] = a[u] * zz;
  }
  // LDS operations of one wave complete in program order; the fence keeps the compiler from moving them
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  double acc = 0.0, acc2 = 0.0;
  {
    const int c1 = CH < len ? CH : len;
    const int hi = rhi < c1 ? rhi : c1;
    int e = rlo + sl;
    for (; e + LR < hi; e += 2 * LR) {
      acc += prod[e];
      acc2 += prod[e + LR];
    }
    if (e < hi) acc += prod[e];
  }
  for (int c0 = CH; c0 < len; c0 += CH) {
    __builtin_amdgcn_wave_barrier();
    const int c1 = (c0 + CH) < len ? (c0 + CH) : len;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int idx = c0 + u * 64 + lane;
      idx = idx < len ? idx : len - 1;
      prod[u * 64 + lane] = vp[idx] * z[cp[idx]];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int lo = rlo > c0 ? rlo : c0;
    const int hi = rhi < c1 ? rhi : c1;
    for (int e = lo + sl; e < hi; e += LR) acc += prod[e - c0];
  }
  acc += acc2;
#pragma unroll
  for (int o = LR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, LR);
  if (mine) {
    const double yv = sg * acc;
    y[(row0 + g) * ldy] = yv;
    if (zout) zout[row0 + g] = sg * yv;  // the next product's operand s o y, scaled here instead of in a pass of its own
  }
}

// Tile shape by the average row length: the register buffer (U*64 entries) should hold an average tile with some room.
static hipError_t launch_spmv_tile(const int64_t* rowptr, const int32_t* col, const double* val, const double* s,
                                   int64_t n, const double* z, double* y, int64_t ldy, double avg_deg,
                                   hipStream_t st, double* zout = nullptr) {
#define SC_LAUNCH_TILE(RW_, U_)                                                                                    \
  do {                                                                                                             \
    const int64_t ntiles = ceil_div64(n, RW_);                                                                     \
    hipLaunchKernelGGL((spmv_tile_kernel<RW_, U_>), dim3((unsigned)ceil_div64(ntiles, kThreads / 64)),              \
                       dim3(kThreads), 0, st, rowptr, col, val, s, z, y, ldy, n, ntiles, zout);                    \
  } while (0)
  const double need = avg_deg * 1.08 / 64.0;  // register slots per lane and row of the tile
  if (need * 32 <= 8) SC_LAUNCH_TILE(32, 8);
  else if (need * 32 <= 12) SC_LAUNCH_TILE(32, 12);
  else if (need * 32 <= 16) SC_LAUNCH_TILE(32, 16);
  else if (need * 32 <= 22) SC_LAUNCH_TILE(32, 22);
  else if (need * 16 <= 22) SC_LAUNCH_TILE(16, 22);
  else SC_LAUNCH_TILE(8, 22);
#undef SC_LAUNCH_TILE
  return hipGetLastError();
}

template <int B>
hipError_t launch_spmm_nz(const int64_t* rowptr, const int32_t* col, const double* val, const double* s, int64_t n,
                          const double* z, double* y, int64_t ldy, double avg_deg, hipStream_t st) {
  if constexpr (B == 1) {
    if (avg_deg >= 6.0) return launch_spmv_tile(rowptr, col, val, s, n, z, y, ldy, avg_deg, st);
  }
  if (avg_deg >= 6.0) {
    // row-block streaming: 64 rows per workgroup for short rows, 32 otherwise (4 or 8 lanes per row sum)
    if (avg_deg < 24.0) {
      hipLaunchKernelGGL((spmm_stream_kernel<B, 64>), dim3(xcd_grid(ceil_div64(n, 64))), dim3(kThreads), 0, st, rowptr,
                         col, val, s, z, y, ldy, n);
    } else {
      hipLaunchKernelGGL((spmm_stream_kernel<B, 32>), dim3(xcd_grid(ceil_div64(n, 32))), dim3(kThreads), 0, st, rowptr,
                         col, val, s, z, y, ldy, n);
    }
    return hipGetLastError();
  }
  int lanes = 4;
  while (lanes < 64 && lanes * 2 <= avg_deg) lanes *= 2;  // largest power of two <= avg_deg, in [4, 64]
#define SC_LAUNCH_NZ(LL)                                                                                       \
  hipLaunchKernelGGL((spmm_nz_kernel<B, LL>), dim3((unsigned)ceil_div64(n, kThreads / LL)), dim3(kThreads), 0, \
                     st, rowptr, col, val, s, z, y, ldy, n)
  switch (lanes) {
    case 4: SC_LAUNCH_NZ(4); break;
    case 8: SC_LAUNCH_NZ(8); break;
    case 16: SC_LAUNCH_NZ(16); break;
    case 32: SC_LAUNCH_NZ(32); break;
    default: SC_LAUNCH_NZ(64); break;
  }
#undef SC_LAUNCH_NZ
  return hipGetLastError();
}

// --------------------------------------------------------------------------------------------
// tall-skinny projection  part = A^T B  (contraction over rows), fp64 MFMA
// --------------------------------------------------------------------------------------------
// A wave owns 64 consecutive A columns and a slice of rows.  Per step of 4 rows lane (i, g) loads
// A[row+g][c0 + 4i .. 4i+3] (32 contiguous bytes) and B[row+g][i (+16)].  MFMA q multiplies the q-th
// of the four A values, so its output row M stands for A column c0 + 4M + q.
template <int NT>
__global__ __launch_bounds__(kThreads) void project_kernel(const double* __restrict__ basis, int64_t n, int64_t ld,
                                                           int acol0, int ja, int bcol0, int b, int rows_per_panel,
                                                           int nwc, int vec_ok, double* __restrict__ part,
                                                           const int* __restrict__ skip) {
  if (skip && *skip) return;  // uniform over the grid: a pass that a device-side test found unnecessary
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int nwr = 4 / nwc;
  const int wc = wave % nwc, wr = wave / nwc;
  const int c0 = ((int)blockIdx.y * nwc + wc) * 64;
  // wave-uniform; happens only with four column tiles per workgroup (nwr = 1), where no barrier follows
  if (c0 >= ja) return;
  const int pidx = (int)blockIdx.x;  // one partial block per workgroup: waves that share a column tile are summed below
  const int sub = rows_per_panel / nwr;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_panel + (int64_t)wr * sub;
  int64_t r1 = r0 + sub;
  if (r1 > n) r1 = n;

  d4 acc[NT][4];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[nt][q] = (d4){0.0, 0.0, 0.0, 0.0};

  const int cbase = c0 + 4 * i;
  const bool full = vec_ok && (cbase + 3 < ja);
  // four row-quads (16 rows) per trip: all their loads are issued before the first MFMA needs them
  constexpr int U = 4;
  int64_t rstart = r0;
  // With all 16 NT block columns present and vector loads allowed, a wave runs the whole trips of its row slice
  // without a branch round any load: the operands of the next trip are requested before the MFMAs of
  // this one (the last request reads the slice's last rows again and is dropped).  With conditional loads the compiler
  // has to wait for every load in flight before the first MFMA, so a wave alternates between loading and multiplying.
  if (vec_ok && ja % 4 == 0 && b == 16 * NT && r1 - r0 >= 4 * U) {  // wave-uniform
    const int64_t rfull = r0 + (r1 - r0) / (4 * U) * (4 * U);
    const int64_t rlast = rfull - 4 * U;  // first row of the last whole trip
    // lanes whose four columns lie past ja read the last four instead: their results are never stored
    const double* __restrict__ abase = basis + acol0 + (cbase + 3 < ja ? cbase : ja - 4);
    const double* __restrict__ bbase = basis + bcol0 + i;
    d4 a0[U], a1[U];
    double v0[U][NT], v1[U][NT];
    auto fetch = [&](d4 (&av)[U], double (&vv)[U][NT], int64_t r) __attribute__((always_inline)) {
      const int64_t rr = r < rlast ? r : rlast;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t row = rr + 4 * u + g;
        av[u] = *reinterpret_cast<const d4*>(abase + row * ld);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) vv[u][nt] = bbase[row * ld + 16 * nt];
      }
    };
    auto mult = [&](const d4 (&av)[U], const double (&vv)[U][NT]) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[nt][q] = MFMA_F64(av[u][q], vv[u][nt], acc[nt][q]);
    };
    fetch(a0, v0, r0);
    for (int64_t r = r0; r < rfull; r += 8 * U) {
      fetch(a1, v1, r + 4 * U);
      mult(a0, v0);
      if (r + 4 * U >= rfull) break;
      fetch(a0, v0, r + 8 * U);
      mult(a1, v1);
    }
    rstart = rfull;
  }
  for (int64_t r = rstart; r < r1; r += 4 * U) {
    double a[U][4];
    double bv[U][NT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t row = r + 4 * u + g;
#pragma unroll
      for (int q = 0; q < 4; ++q) a[u][q] = 0.0;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bv[u][nt] = 0.0;
      if (row < r1) {
        const double* rp = basis + row * ld;
        const double* ap = rp + acol0 + cbase;
        if (full) {
          const d4 v = *reinterpret_cast<const d4*>(ap);
          a[u][0] = v[0]; a[u][1] = v[1]; a[u][2] = v[2]; a[u][3] = v[3];
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (cbase + q < ja) a[u][q] = ap[q];
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          if (i + 16 * nt < b) bv[u][nt] = rp[bcol0 + i + 16 * nt];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[nt][q] = MFMA_F64(a[u][q], bv[u][nt], acc[nt][q]);
  }

  if (nwr > 1) {
    // Few basis columns: the workgroup's waves have taken row slices of the same column tile.  Their sums are added
    // here, in wave order, instead of being written as partial blocks of their own: with one partial block per wave
    // the limit on partial blocks left a short contraction with two waves per compute unit.
    extern __shared__ double red[];  // (nwr - 1) * nwc slots of 16 * NT values per lane
    constexpr int SLOT = 16 * NT * 64;
    if (wr > 0) {
      double* mine = red + (size_t)((wr - 1) * nwc + wc) * SLOT + lane;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) mine[((nt * 4 + q) * 4 + rr) * 64] = acc[nt][q][rr];
    }
    __syncthreads();
    if (wr > 0) return;
    for (int w = 1; w < nwr; ++w) {
      const double* theirs = red + (size_t)((w - 1) * nwc + wc) * SLOT + lane;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) acc[nt][q][rr] += theirs[((nt * 4 + q) * 4 + rr) * 64];
    }
  }
  double* out = part + (int64_t)pidx * ja * kPartialPad;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int c = c0 + 4 * (4 * rr + g) + q;
        if (c < ja) out[(int64_t)c * kPartialPad + i + 16 * nt] = acc[nt][q][rr];
      }
}

// One output element per 32 threads: thread (e, r) sums the partials p = r*chunk .. (r+1)*chunk-1 in
// order, then the 32 sub-sums are added in the fixed order r = 0..31, so the result does not depend on
// scheduling.  Only the b meaningful columns of every kPartialPad-wide row are touched.
constexpr int kRedSplit = 32;
constexpr int kRedElems = kThreads / kRedSplit;  // 32 output elements per workgroup
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const double* __restrict__ part, int npart, int ja,
                                                                   int ncol, double* __restrict__ h,
                                                                   double* __restrict__ hsum, int accumulate,
                                                                   double* __restrict__ slot, int slot_row0,
                                                                   const int* __restrict__ skip) {
  __shared__ double sub[kRedSplit][kRedElems + 1];
  if (skip && *skip) return;  // uniform over the grid
  const int el = threadIdx.x % kRedElems, r = threadIdx.x / kRedElems;
  const int e = blockIdx.x * kRedElems + el;  // element index over ja * ncol
  const int total = ja * ncol;
  const int c = e / ncol, t = e - c * ncol;
  double acc = 0.0;
  if (e < total) {
    const int chunk = (npart + kRedSplit - 1) / kRedSplit;
    const int p0 = r * chunk;
    int p1 = p0 + chunk;
    if (p1 > npart) p1 = npart;
    const int64_t stride = (int64_t)ja * kPartialPad;
    const double* p = part + (int64_t)c * kPartialPad + t;
    int q = p0;
    for (; q + 8 <= p1; q += 8) {  // eight independent loads in flight, added in index order
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(q + u) * stride];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; q < p1; ++q) acc += p[q * stride];
  }
  sub[r][el] = acc;
  __syncthreads();
  if (r == 0 && e < total) {
    double tot = sub[0][el];
#pragma unroll
    for (int q = 1; q < kRedSplit; ++q) tot += sub[q][el];
    const int idx = c * kPartialPad + t;
    if (h) h[idx] = tot;
    if (hsum) {
      if (accumulate) tot += hsum[idx];
      hsum[idx] = tot;
    }
    if (slot && c >= slot_row0) slot[(c - slot_row0) * kPartialPad + t] = tot;
  }
}

// The coefficient chunk bmat[k0 : k0+kc, n0 : n0+NT*16] (row-major, leading dimension ldb; columns from ncols on
// and rows from kc to kc16 count as zero) goes into LDS in the order the MFMA operand reads want: the 64 lanes of one
// MFMA read 64 consecutive doubles.  Every thread first requests a batch of 16 of its elements, with clamped
// addresses instead of tests round the loads, and only then parks them: one memory latency per batch of 4,096
// elements.  (Written as a loop of load, test, store per element, the compiler waits for each load before the next
// is requested: 16 latencies per chunk, more than the chunk's MFMAs take.)
template <int NT>
__device__ __forceinline__ void stage_coefficients(double* __restrict__ lds, const double* __restrict__ bmat,
                                                   int64_t ldb, int k0, int kc, int kc16, int n0, int ncols) {
  constexpr int BW = NT * 16;
  constexpr int BATCH = 16;
  for (int base = 0; base < kc16 * BW; base += kThreads * BATCH) {  // uniform; the LDS chunk holds whole batches
    double v[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int e = base + u * kThreads + (int)threadIdx.x;
      const int kk = e / BW, t = e % BW;
      const int kr = kk < kc ? kk : kc - 1;
      const int tc = n0 + t < ncols ? n0 + t : ncols - 1;
      v[u] = bmat[(int64_t)(k0 + kr) * ldb + tc];
    }
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      const int e = base + u * kThreads + (int)threadIdx.x;
      const int kk = e / BW, t = e % BW;
      const int kt = kk >> 4, rem = kk & 15, gg = rem >> 2, q = rem & 3;
      const int nt = t >> 4, ii = t & 15;
      lds[((((kt * 4 + q) * NT + nt) * 4 + gg) << 4) + ii] = (kk < kc && n0 + t < ncols) ? v[u] : 0.0;
    }
  }
}

// --------------------------------------------------------------------------------------------
// row GEMM  C = A * Bm  (contraction over basis columns), fp64 MFMA, Bm staged through LDS
// --------------------------------------------------------------------------------------------
// A wave owns MT*16 rows and NT*16 output columns.  Per step of 16 contraction indices lane (i, g)
// loads A[row0+i][k + 4g .. 4g+3]; MFMA q contracts over the indices k + 4g + q, g = 0..3.  The Bm
// chunk sits in LDS permuted so that the 64 lanes of one MFMA read 64 consecutive doubles.
// PIPE: loads one trip ahead of the MFMAs, for long contractions only (see update_gram_kernel).
template <int NT, int MT, bool PIPE>
__global__ __launch_bounds__(kThreads) void row_gemm_kernel(double* __restrict__ basis, int64_t n, int64_t ld,
                                                            int acol0, int kdim, const double* __restrict__ bmat,
                                                            int ldb, int ncols, int mode, int ccol0,
                                                            double* __restrict__ out, int64_t ldo, int vec_ok,
                                                            const int32_t* __restrict__ rowmap,
                                                            const int* __restrict__ skip) {
  if (skip && *skip) return;  // uniform over the grid
  constexpr int KC = 4096 / (NT * 16);  // contraction indices per LDS chunk (32 KB)
  __shared__ double lds[KC * NT * 16];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int n0 = (int)blockIdx.y * NT * 16;
  const int64_t row0 = ((int64_t)blockIdx.x * 4 + wave) * (16 * MT);

  d4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (d4){0.0, 0.0, 0.0, 0.0};
  d4 a0[2][MT], a1[2][MT];  // operand registers of the pipelined path: a0 carries over from chunk to chunk

  for (int k0 = 0; k0 < kdim; k0 += KC) {
    const int kc = (kdim - k0) < KC ? (kdim - k0) : KC;
    const int kc16 = (kc + 15) & ~15;
    __syncthreads();
    stage_coefficients<NT>(lds, bmat, ldb, k0, kc, kc16, n0, ncols);
    __syncthreads();
    int kk0 = 0;
    // A wave whose rows all exist runs the trips of the chunk without a branch round any load: the operands of the
    // next trip are requested before the MFMAs of this one (the last request repeats the last trip's and is dropped);
    // columns past kdim are read from the last four instead: their B rows in LDS are zero (or skipped).
    if (PIPE && vec_ok && row0 + 16 * MT <= n && kdim % 4 == 0) {  // wave-uniform
      const double* __restrict__ abase = basis + (row0 + i) * ld + acol0;
      // The request that follows a chunk's last trip is the first trip of the NEXT chunk (columns are clamped to the
      // contraction's end, not to the chunk's): it is in flight while the workgroup restages the coefficient chunk
      // behind two barriers, so the stream of operand loads no longer drains at every chunk boundary.
      auto fetch = [&](d4 (&av)[2][MT], int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          int kcol = k0 + kb + 16 * h + 4 * g;
          kcol = kcol + 3 < kdim ? kcol : kdim - 4;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            av[h][mt] = *reinterpret_cast<const d4*>(abase + (int64_t)mt * 16 * ld + kcol);
        }
      };
      auto mult = [&](const d4 (&av)[2][MT], int kb) __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          if (kb + 16 * h < kc16) {  // uniform; the LDS slots beyond kc16 were not filled
            const int kt = (kb >> 4) + h;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int nt = 0; nt < NT; ++nt) {
                const double bq = lds[((((kt * 4 + q) * NT + nt) * 4 + g) << 4) + i];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = MFMA_F64(av[h][mt][q], bq, acc[mt][nt]);
              }
          }
        }
      };
      if (k0 == 0) fetch(a0, 0);  // later chunks find their first trip requested by the chunk before
      for (int kb = 0; kb < kc16; kb += 64) {
        fetch(a1, kb + 32);
        mult(a0, kb);
        if (kb + 32 >= kc16) break;
        fetch(a0, kb + 64);
        mult(a1, kb + 32);
      }
      kk0 = kc16;
    }
    // two 16-index groups per trip: their loads are issued together, ahead of the MFMAs that use them
    for (int kk = kk0; kk < kc16; kk += 32) {
      double a[2][MT][4];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int kcol = k0 + kk + 16 * h + 4 * g;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int64_t row = row0 + mt * 16 + i;
#pragma unroll
          for (int q = 0; q < 4; ++q) a[h][mt][q] = 0.0;
          if (row < n && kk + 16 * h < kc16) {
            const double* ap = basis + row * ld + acol0 + kcol;
            if (vec_ok && kcol + 3 < kdim) {
              const d4 v = *reinterpret_cast<const d4*>(ap);
              a[h][mt][0] = v[0]; a[h][mt][1] = v[1]; a[h][mt][2] = v[2]; a[h][mt][3] = v[3];
            } else {
#pragma unroll
              for (int q = 0; q < 4; ++q)
                if (kcol + q < kdim) a[h][mt][q] = ap[q];
            }
          }
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (kk + 16 * h < kc16) {  // uniform; the LDS slots beyond kc16 were not filled
          const int kt = (kk >> 4) + h;
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              const double bq = lds[((((kt * 4 + q) * NT + nt) * 4 + g) << 4) + i];
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = MFMA_F64(a[h][mt][q], bq, acc[mt][nt]);
            }
        }
      }
    }
  }

#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int64_t row = row0 + mt * 16 + 4 * rr + g;
        const int t = n0 + nt * 16 + i;
        if (row < n && t < ncols) {
          const double v = acc[mt][nt][rr];
          if (mode == 0) {
            basis[row * ld + ccol0 + t] -= v;
          } else if (mode == 3) {
            basis[row * ld + ccol0 + t] = v;
          } else if (mode == 1) {
            out[row * ldo + t] = v;
          } else {
            out[(int64_t)t * ldo + (rowmap ? (int64_t)rowmap[row] : row)] = v;
          }
        }
      }
}

// --------------------------------------------------------------------------------------------
// block orthonormalization helpers
// --------------------------------------------------------------------------------------------
constexpr int kCholThreads = 64;  // one wave: its barriers cost next to nothing
__global__ __launch_bounds__(kCholThreads) void gram_cholesky_kernel(const double* __restrict__ g_in, int b,
                                                                 double* __restrict__ g_out,
                                                                 double* __restrict__ rinv_out,
                                                                 double* __restrict__ r_out,
                                                                 const double* __restrict__ rprev, double abs_tol2,
                                                                 double rel_tol) {
  __shared__ double G[kMaxBlock][kMaxBlock + 1];
  __shared__ double R[kMaxBlock][kMaxBlock + 1];
  __shared__ double Ri[kMaxBlock][kMaxBlock + 1];
  __shared__ int dropped;
  const int tid = threadIdx.x;
  for (int e = tid; e < b * b; e += kCholThreads) {
    const int c = e / b, t = e % b;
    G[c][t] = g_in[c * kPartialPad + t];
    R[c][t] = 0.0;
    Ri[c][t] = 0.0;
  }
  __syncthreads();
  if (g_out)
    for (int e = tid; e < b * b; e += kCholThreads) {
      const int c = e / b, t = e % b;
      g_out[c * kPartialPad + t] = c <= t ? G[c][t] : G[t][c];  // mirror the upper triangle
    }
  // Cholesky G = R^T R on the upper triangle, dropping dependent columns
  for (int k = 0; k < b; ++k) {
    if (tid == 0) {
      double p = G[k][k];
      for (int q = 0; q < k; ++q) p -= R[q][k] * R[q][k];
      const bool drop = !(G[k][k] > abs_tol2) || !(p > rel_tol * G[k][k]);
      dropped = drop ? 1 : 0;
      R[k][k] = drop ? 0.0 : sqrt(p);
    }
    __syncthreads();
    if (tid > k && tid < b && !dropped) {
      double v = G[k][tid];
      for (int q = 0; q < k; ++q) v -= R[q][k] * R[q][tid];
      R[k][tid] = v / R[k][k];
    }
    __syncthreads();
  }
  // inverse of R on the kept columns, one thread per column
  if (tid < b) {
    const int c = tid;
    if (R[c][c] != 0.0) {
      Ri[c][c] = 1.0 / R[c][c];
      for (int r = c - 1; r >= 0; --r) {
        if (R[r][r] == 0.0) continue;
        double v = 0.0;
        for (int t = r + 1; t <= c; ++t) v += R[r][t] * Ri[t][c];
        Ri[r][c] = -v / R[r][r];
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < b * b; e += kCholThreads) {
    const int c = e / b, t = e % b;
    if (rinv_out) rinv_out[c * kPartialPad + t] = Ri[c][t];
    if (r_out) {
      double v = R[c][t];
      if (rprev) {
        v = 0.0;
        for (int q = c; q < b; ++q) v += R[c][q] * rprev[q * kPartialPad + t];
      }
      r_out[c * kPartialPad + t] = v;
    }
  }
}

constexpr int kRinvTrips = 16;  // row groups per workgroup: the staging of R^-1 is paid once for all of them
__global__ __launch_bounds__(kThreads) void apply_rinv_kernel(double* __restrict__ basis, int64_t n, int64_t ld,
                                                              int col0, int b, const double* __restrict__ rinv,
                                                              double* __restrict__ z, const double* __restrict__ s) {
  __shared__ double Ri[kMaxBlock][kMaxBlock + 1];
  __shared__ double Wt[2 * kThreads];  // rows_per_block rows of b + 1 doubles (b >= 1)
  for (int e = threadIdx.x; e < b * b; e += kThreads) Ri[e / b][e % b] = rinv[(e / b) * kPartialPad + (e % b)];
  const int rows_per_block = kThreads / b;
  const int t = threadIdx.x % b, rl = threadIdx.x / b;
  // the entry of the next trip is requested before this trip's sums, so its latency hides behind them
  const int64_t first = (int64_t)blockIdx.x * kRinvTrips * rows_per_block + rl;
  double ahead = first < n ? basis[first * ld + col0 + t] : 0.0;
  for (int trip = 0; trip < kRinvTrips; ++trip) {
    const int64_t row = ((int64_t)blockIdx.x * kRinvTrips + trip) * rows_per_block + rl;
    __syncthreads();  // the tile of the trip before has been read (and, first time round, R^-1 is staged)
    Wt[rl * (b + 1) + t] = ahead;
    __syncthreads();
    const int64_t nrow = row + rows_per_block;
    ahead = (trip + 1 < kRinvTrips && nrow < n) ? basis[nrow * ld + col0 + t] : 0.0;
    double acc = 0.0;
    for (int q = 0; q <= t; ++q) acc += Wt[rl * (b + 1) + q] * Ri[q][t];
    if (row < n) {
      basis[row * ld + col0 + t] = acc;
      if (z) z[row * b + t] = s ? s[row] * acc : acc;
    }
  }
}

// --------------------------------------------------------------------------------------------
// misc
// --------------------------------------------------------------------------------------------
__device__ inline uint64_t mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

__global__ __launch_bounds__(kThreads) void random_block_kernel(double* __restrict__ basis, int64_t n, int64_t ld,
                                                                int col0, int b, uint64_t seed, uint64_t stream_id) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * b) return;
  const int64_t i = idx / b;
  const int t = (int)(idx - i * b);
  const uint64_t h = mix64(mix64(seed ^ (stream_id * 0xD1B54A32D192ED03ull)) + (uint64_t)idx);
  const double u = (double)(h >> 11) * (1.0 / 9007199254740992.0);  // [0, 1)
  basis[i * ld + col0 + t] = 2.0 * u - 1.0;
}

// dst[i, dcol0 + t] -= src[i, scol0 + t], t < w
__global__ __launch_bounds__(kThreads) void sub_cols_kernel(const double* __restrict__ src, int64_t lds, int scol0,
                                                            double* __restrict__ dst, int64_t ldd, int dcol0, int w,
                                                            int64_t n) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * w) return;
  const int64_t i = idx / w;
  const int t = (int)(idx - i * w);
  dst[i * ldd + dcol0 + t] -= src[i * lds + scol0 + t];
}

// basis[i, col] = v[r(i)]: one column of the row-major basis from a plain vector in the caller's numbering
// (r(i) = rowmap[i], the original index of internal row i, if rowmap is given, else i)
__global__ __launch_bounds__(kThreads) void set_column_kernel(double* __restrict__ basis, int64_t n, int64_t ld, int col,
                                                              const double* __restrict__ v,
                                                              const int32_t* __restrict__ rowmap) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n) return;
  basis[i * ld + col] = v[rowmap ? (int64_t)rowmap[i] : i];
}

__global__ __launch_bounds__(kThreads) void copy_cols_kernel(const double* __restrict__ src, int64_t lds, int scol0,
                                                             double* __restrict__ dst, int64_t ldd, int dcol0, int w,
                                                             int64_t n) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * w) return;
  const int64_t i = idx / w;
  const int t = (int)(idx - i * w);
  dst[i * ldd + dcol0 + t] = src[i * lds + scol0 + t];
}

// out[pos[c] * n + o] = basis[r(o) * ld + c] for the basis columns c < ncols with pos[c] >= 0: selected columns of the
// row-major basis, written column-major in the caller's row numbering (r(o) = inv[o], the internal row of original
// row o, if inv is given, else o).  A workgroup moves a 64 x 64 tile through LDS: the reads take 512 contiguous bytes
// of each basis row (consecutive basis columns), the writes 512 contiguous bytes of each output column (consecutive
// original rows); only whole rows and whole columns are permuted, never single elements.
__global__ __launch_bounds__(kThreads) void gather_cols_colmajor_kernel(const double* __restrict__ basis, int64_t n,
                                                                        int64_t ld, const int32_t* __restrict__ pos,
                                                                        int ncols, double* __restrict__ out,
                                                                        const int32_t* __restrict__ inv) {
  __shared__ double tile[64][65];
  const int64_t i0 = (int64_t)blockIdx.x * 64;
  const int c0 = blockIdx.y * 64;
  // thread (c, rq) takes column c0 + c of the rows i0 + rq + 4u, u < 16.  All sixteen source rows are looked up, then
  // all sixteen basis entries requested, with clamped addresses instead of tests round the loads, and only then
  // parked: two memory latencies per tile (written as one loop of look-up, load and store the compiler waits for
  // every load before it requests the next: thirty-two latencies).
  const int c = threadIdx.x % 64, rq = threadIdx.x / 64;
  const int cc = c0 + c < ncols ? c0 + c : ncols - 1;
  int64_t src[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int64_t row = i0 + rq + 4 * u < n ? i0 + rq + 4 * u : n - 1;
    src[u] = inv ? (int64_t)inv[row] : row;
  }
  double v[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) v[u] = basis[src[u] * ld + cc];
#pragma unroll
  for (int u = 0; u < 16; ++u) tile[c][rq + 4 * u] = v[u];
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * 64; idx += kThreads) {
    const int oc = idx / 64, r = idx % 64;
    if (i0 + r < n && c0 + oc < ncols) {
      const int p = pos[c0 + oc];
      if (p >= 0) out[(int64_t)p * n + i0 + r] = tile[oc][r];
    }
  }
}

// out[t * n + o] *= s[r(o)] for t < k: column-major vectors in the caller's numbering times the scaling vector held in
// the internal numbering (r(o) = inv[o] if inv is given, else o).
__global__ __launch_bounds__(kThreads) void scale_rows_colmajor_kernel(double* __restrict__ out, int64_t n, int k,
                                                                       const double* __restrict__ s,
                                                                       const int32_t* __restrict__ inv) {
  const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= n) return;
  const double f = s[inv ? (int64_t)inv[o] : o];
  for (int t = 0; t < k; ++t) out[(int64_t)t * n + o] *= f;
}

// Row o of the n x k column-major matrix out (the embedding of node o) is scaled to unit 2-norm; a zero row stays zero.
__global__ __launch_bounds__(kThreads) void normalize_rows_colmajor_kernel(double* __restrict__ out, int64_t n, int k) {
  const int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (o >= n) return;
  double ss = 0.0;
  for (int t = 0; t < k; ++t) {
    const double v = out[(int64_t)t * n + o];
    ss += v * v;
  }
  if (ss > 0.0) {
    const double f = 1.0 / sqrt(ss);
    for (int t = 0; t < k; ++t) out[(int64_t)t * n + o] *= f;
  }
}

// One step of the three-term Chebyshev recurrence on packed n x b blocks (leading dimension b):
//   ynext = alpha * (w - shift * ycur) - beta * yprev,   znext = s o ynext   (the packed operand of the next product)
// ynext may be the buffer of yprev (each element is read before it is written by the same thread).
__global__ __launch_bounds__(kThreads) void cheb_combine_kernel(const double* __restrict__ w,
                                                                const double* __restrict__ ycur, const double* yprev,
                                                                const double* __restrict__ s, double alpha,
                                                                double shift, double beta, double* ynext,
                                                                double* __restrict__ znext, int64_t n, int b) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * b) return;
  double v = alpha * (w[idx] - shift * ycur[idx]);
  if (beta != 0.0) v -= beta * yprev[idx];
  ynext[idx] = v;
  znext[idx] = s[idx / b] * v;
}

// --------------------------------------------------------------------------------------------
// fused pieces of the block step
// --------------------------------------------------------------------------------------------
// Second CGS2 update fused with the Gram matrix of the updated block:
//   basis[:, ccol0 : ccol0+b] -= basis[:, acol0 : acol0+kdim] * bmat,   gpart[blockIdx.x] = sum over this
//   workgroup's rows of W_new^T W_new.
// overwrite != 0: the product replaces the block instead of being subtracted from it.  With acol0 = ccol0, kdim = b
// and bmat = R^-1 this is the scaling pass W <- W R^-1 of the Cholesky QR (a wave reads its own 32 rows of the
// block completely before it writes them).
// Workgroups walk the 128-row tiles with a grid stride, so the number of Gram partials is the grid size.
// PIPE: the variant for long contractions, see the note at its loop.  It needs more registers (fewer resident waves),
// which costs more than it gains when the contraction has only a trip or two, so it is a kernel of its own.
template <int NT, bool PIPE>
__global__ __launch_bounds__(kThreads) void update_gram_kernel(double* __restrict__ basis, int64_t n, int64_t ld,
                                                               int acol0, int kdim, const double* __restrict__ bmat, int b,
                                                               int ccol0, int vec_ok, int overwrite,
                                                               double* __restrict__ gpart,
                                                               const int* __restrict__ skip) {
  if (skip && *skip) return;  // uniform over the grid
  constexpr int MT = 2;
  constexpr int BW = NT * 16;
  constexpr int KC = 4096 / BW;
  constexpr int WP = NT == 1 ? BW + 1 : BW;  // row pitch of the tile of new block rows
  __shared__ double lds[KC * BW];
  __shared__ double wt[128 * WP];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, g = lane >> 4;
  const int64_t ntiles = (n + 127) / 128;
  const bool single = kdim <= KC;

  auto load_chunk = [&](int k0, int kc, int kc16) {
    stage_coefficients<NT>(lds, bmat, kPartialPad, k0, kc, kc16, 0, b);
  };
  if (single) {
    load_chunk(0, kdim, (kdim + 15) & ~15);
    __syncthreads();
  }

  d4 gacc[NT][NT];
#pragma unroll
  for (int x = 0; x < NT; ++x)
#pragma unroll
    for (int y = 0; y < NT; ++y) gacc[x][y] = (d4){0.0, 0.0, 0.0, 0.0};

  for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int64_t row0 = (tile * 4 + wave) * (16 * MT);
    d4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (d4){0.0, 0.0, 0.0, 0.0};
    for (int k0 = 0; k0 < kdim; k0 += KC) {
      const int kc = (kdim - k0) < KC ? (kdim - k0) : KC;
      const int kc16 = (kc + 15) & ~15;
      if (!single) {
        __syncthreads();
        load_chunk(k0, kc, kc16);
        __syncthreads();
      }
      int kk0 = 0;
      // A wave whose 32 rows all exist runs the trips of the chunk without a branch round any load: the operands of
      // the next trip are requested before the MFMAs of this one (the last request repeats the last trip's and is
      // dropped).  Behind conditional loads the compiler waits for every load in flight before the
      // first MFMA.
      if (PIPE && vec_ok && row0 + 16 * MT <= n && kdim % 4 == 0) {  // wave-uniform
        const int klast = (kc16 - 1) / 32 * 32;  // start of the chunk's last trip
        const double* __restrict__ abase = basis + (row0 + i) * ld + acol0;
        d4 a0[2][MT], a1[2][MT];
        // columns past kdim are read from the last four instead: their B rows in LDS are zero (or skipped)
        auto fetch = [&](d4 (&av)[2][MT], int kb) __attribute__((always_inline)) {
          const int kq = kb < klast ? kb : klast;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            int kcol = k0 + kq + 16 * h + 4 * g;
            kcol = kcol + 3 < kdim ? kcol : kdim - 4;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
              av[h][mt] = *reinterpret_cast<const d4*>(abase + (int64_t)mt * 16 * ld + kcol);
          }
        };
        auto mult = [&](const d4 (&av)[2][MT], int kb) __attribute__((always_inline)) {
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            if (kb + 16 * h < kc16) {  // uniform; the LDS slots beyond kc16 were not filled
              const int kt = (kb >> 4) + h;
#pragma unroll
              for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                  const double bq = lds[((((kt * 4 + q) * NT + nt) * 4 + g) << 4) + i];
#pragma unroll
                  for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = MFMA_F64(av[h][mt][q], bq, acc[mt][nt]);
                }
            }
          }
        };
        fetch(a0, 0);
        for (int kb = 0; kb < kc16; kb += 64) {
          fetch(a1, kb + 32);
          mult(a0, kb);
          if (kb + 32 >= kc16) break;
          fetch(a0, kb + 64);
          mult(a1, kb + 32);
        }
        kk0 = kc16;
      }
      // two 16-index groups per trip: their loads are issued together, ahead of the MFMAs that use them
      for (int kk = kk0; kk < kc16; kk += 32) {
        double a[2][MT][4];
  #pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int kcol = k0 + kk + 16 * h + 4 * g;
  #pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int64_t row = row0 + mt * 16 + i;
  #pragma unroll
            for (int q = 0; q < 4; ++q) a[h][mt][q] = 0.0;
            if (row < n && kk + 16 * h < kc16) {
              const double* ap = basis + row * ld + acol0 + kcol;
              if (vec_ok && kcol + 3 < kdim) {
                const d4 v = *reinterpret_cast<const d4*>(ap);
                a[h][mt][0] = v[0]; a[h][mt][1] = v[1]; a[h][mt][2] = v[2]; a[h][mt][3] = v[3];
              } else {
  #pragma unroll
                for (int q = 0; q < 4; ++q)
                  if (kcol + q < kdim) a[h][mt][q] = ap[q];
              }
            }
          }
        }
  #pragma unroll
        for (int h = 0; h < 2; ++h) {
          if (kk + 16 * h < kc16) {  // uniform; the LDS slots beyond kc16 were not filled
            const int kt = (kk >> 4) + h;
  #pragma unroll
            for (int q = 0; q < 4; ++q)
  #pragma unroll
              for (int nt = 0; nt < NT; ++nt) {
                const double bq = lds[((((kt * 4 + q) * NT + nt) * 4 + g) << 4) + i];
  #pragma unroll
                for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = MFMA_F64(a[h][mt][q], bq, acc[mt][nt]);
              }
          }
        }
      }
    }
    // new block rows: to memory and into the tile
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int lr = wave * 32 + mt * 16 + 4 * rr + g;
          const int64_t row = row0 + mt * 16 + 4 * rr + g;
          const int t = nt * 16 + i;
          double nv = 0.0;
          if (row < n && t < b) {
            double* p = basis + row * ld + ccol0 + t;
            nv = overwrite == 1 ? acc[mt][nt][rr] : *p - acc[mt][nt][rr];
            if (overwrite != 2) *p = nv;  // 2: only the Gram matrix of the updated block is wanted
          }
          wt[lr * WP + t] = nv;
        }
    __syncthreads();
    // Gram of this wave's 32 rows: contraction over rows, 4 rows per MFMA
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const int lr = wave * 32 + ks * 4 + g;
      double av[NT];
#pragma unroll
      for (int x = 0; x < NT; ++x) av[x] = wt[lr * WP + i + 16 * x];
#pragma unroll
      for (int x = 0; x < NT; ++x)
#pragma unroll
        for (int y = 0; y < NT; ++y) gacc[x][y] = MFMA_F64(av[x], av[y], gacc[x][y]);
    }
    __syncthreads();
  }
  // the four waves' Gram blocks are added in wave order
  __syncthreads();
#pragma unroll
  for (int x = 0; x < NT; ++x)
#pragma unroll
    for (int y = 0; y < NT; ++y)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int c1 = 16 * x + 4 * rr + g, c2 = 16 * y + i;
        lds[(wave * BW + c1) * BW + c2] = gacc[x][y][rr];
      }
  __syncthreads();
  for (int e = threadIdx.x; e < BW * BW; e += kThreads) {
    const int c1 = e / BW, c2 = e % BW;
    if (c1 < b && c2 < b) {
      double tot = lds[c1 * BW + c2];
#pragma unroll
      for (int w = 1; w < 4; ++w) tot += lds[(w * BW + c1) * BW + c2];
      gpart[((int64_t)blockIdx.x * b + c1) * kPartialPad + c2] = tot;
    }
  }
}

// Cholesky of the b x b Gram matrix in the registers of one wave: lane t owns column t of G, R and R^-1;
// values of other columns travel by lane reads.  Same dropping rule as documented in kernels.h.
// Value of lane `l` (a compile-time constant after unrolling) for the whole wave: a scalar lane read, not a trip
// through the LDS crossbar.
__device__ __forceinline__ double bcast_lane(double v, int l) {
  const long long bits = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane((int)bits, l);
  const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), l);
  return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

template <int B>
__global__ __launch_bounds__(64) void chol_reg_kernel(const double* __restrict__ g_in, double* __restrict__ g_out,
                                                      double* __restrict__ rinv_out, double* __restrict__ r_out,
                                                      const double* __restrict__ rprev, double abs_tol2,
                                                      double rel_tol) {
  const int t = threadIdx.x;
  const bool act = t < B;
  const int tc = act ? t : 0;
  double gcol[B], rcol[B], ricol[B];
#pragma unroll
  for (int q = 0; q < B; ++q) {
    const int lo = q < tc ? q : tc, hi = q < tc ? tc : q;
    gcol[q] = g_in[lo * kPartialPad + hi];  // upper triangle, mirrored
    rcol[q] = 0.0;
    ricol[q] = 0.0;
  }
  if (g_out && act) {
#pragma unroll
    for (int q = 0; q < B; ++q) g_out[q * kPartialPad + t] = gcol[q];
  }
#pragma unroll
  for (int k = 0; k < B; ++k) {
    double v = gcol[k];
#pragma unroll
    for (int q = 0; q < k; ++q) v -= bcast_lane(rcol[q], k) * rcol[q];
    const double gkk = bcast_lane(gcol[k], k), pk = bcast_lane(v, k);
    const bool drop = !(gkk > abs_tol2) || !(pk > rel_tol * gkk);
    const double rkk = drop ? 0.0 : sqrt(pk);
    rcol[k] = (t == k) ? rkk : ((t > k && !drop) ? v / rkk : 0.0);
  }
  double rcc = 0.0;  // own diagonal entry
#pragma unroll
  for (int q = 0; q < B; ++q) rcc = (q == t) ? rcol[q] : rcc;
#pragma unroll
  for (int r = B - 1; r >= 0; --r) {
    const double rrr = bcast_lane(rcol[r], r);
    double sum = 0.0;
#pragma unroll
    for (int x = r + 1; x < B; ++x) {
      const double rrx = bcast_lane(rcol[r], x);
      sum += (x <= t) ? rrx * ricol[x] : 0.0;
    }
    double v = 0.0;
    if (rrr != 0.0 && rcc != 0.0) v = (t == r) ? 1.0 / rrr : (t > r ? -sum / rrr : 0.0);
    ricol[r] = v;
  }
  if (rinv_out && act) {
#pragma unroll
    for (int q = 0; q < B; ++q) rinv_out[q * kPartialPad + t] = ricol[q];
  }
  if (r_out) {
    double pcol[B];
    if (rprev) {
#pragma unroll
      for (int x = 0; x < B; ++x) pcol[x] = rprev[x * kPartialPad + tc];
    }
#pragma unroll
    for (int q = 0; q < B; ++q) {
      double v = rcol[q];
      if (rprev) {
        v = 0.0;
#pragma unroll
        for (int x = q; x < B; ++x) v += bcast_lane(rcol[q], x) * pcol[x];
      }
      if (act) r_out[q * kPartialPad + t] = v;
    }
  }
}


// --------------------------------------------------------------------------------------------
// connected components by minimum-label propagation, and the row/column permutation of the CSR
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void iota_kernel(int32_t* __restrict__ label, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) label[i] = (int32_t)i;
}

// One round: label[i] <- min over i and its neighbours (entries with weight exactly 0 do not connect), followed
// by pointer jumping label <- label[label].  Labels only decrease and always name a node of the same component,
// so concurrent in-place updates are harmless; *changed is set if anything moved.
__global__ __launch_bounds__(kThreads) void cc_round_kernel(const int64_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ col,
                                                            const double* __restrict__ val, int32_t* label, int64_t n,
                                                            int* __restrict__ changed) {
  const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 4;
  const int lane = threadIdx.x & 15;
  if (row >= n) return;  // uniform over the 16-lane group
  const int32_t mine = label[row];
  int32_t m = mine;
  const int64_t e1 = rowptr[row + 1];
  for (int64_t e = rowptr[row] + lane; e < e1; e += 16) {
    if (val[e] != 0.0) {
      const int32_t l = label[col[e]];
      m = l < m ? l : m;
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) {
    const int32_t other = __shfl_xor(m, o, 16);
    m = other < m ? other : m;
  }
  if (lane == 0) {
    for (int hop = 0; hop < 64; ++hop) {  // labels strictly decrease along the chain
      const int32_t up = label[m];
      if (up >= m) break;
      m = up;
    }
    if (m < mine) {
      label[row] = m;
      *changed = 1;
    }
  }
}

// Row p of the permuted matrix is row old_of_new[p] of the input with columns renamed by new_of_old.
__global__ __launch_bounds__(kThreads) void permute_csr_kernel(const int64_t* __restrict__ rowptr,
                                                               const int32_t* __restrict__ col,
                                                               const double* __restrict__ val,
                                                               const int32_t* __restrict__ old_of_new,
                                                               const int32_t* __restrict__ new_of_old,
                                                               const int64_t* __restrict__ rowptr_new,
                                                               int32_t* __restrict__ col_new,
                                                               double* __restrict__ val_new, int64_t n) {
  const int64_t p = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 4;
  const int lane = threadIdx.x & 15;
  if (p >= n) return;
  const int64_t old = old_of_new[p];
  const int64_t src = rowptr[old], len = rowptr[old + 1] - src, dst = rowptr_new[p];
  for (int64_t t = lane; t < len; t += 16) {
    col_new[dst + t] = new_of_old[col[src + t]];
    val_new[dst + t] = val[src + t];
  }
}

// basis[i, col0 + t] = (label of row i == t-th wanted label) ? sqrt(d_i / vol) : 0, written from per-row data:
// comp[i] in [0, ncomp) is the component of (permuted) row i, coef[i] = sqrt(d_i / vol(comp[i])).
__global__ __launch_bounds__(kThreads) void nullspace_fill_kernel(double* __restrict__ basis, int64_t n, int64_t ld,
                                                                  int col0, int ncols, const int32_t* __restrict__ comp,
                                                                  const double* __restrict__ coef) {
  const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= n * ncols) return;
  const int64_t i = idx / ncols;
  const int t = (int)(idx - i * ncols);
  basis[i * ld + col0 + t] = comp[i] == t ? coef[i] : 0.0;
}

}  // namespace

// ============================================================================================
// launch wrappers
// ============================================================================================
hipError_t launch_validate_csr(const int64_t* rowptr, const int32_t* col, int64_t n, int64_t nnz, int* flag,
                               hipStream_t st) {
  hipLaunchKernelGGL(validate_rowptr_kernel, dim3((unsigned)ceil_div64(n, kThreads)), dim3(kThreads), 0, st, rowptr,
                     n, nnz, flag);
  if (nnz > 0) {
    int64_t blocks = ceil_div64(nnz, kThreads);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(validate_col_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, col, nnz, n, flag);
  }
  return hipGetLastError();
}

hipError_t launch_validate_symmetry(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, int* flag,
                                    hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(validate_symmetry_kernel, dim3((unsigned)ceil_div64(n * 64, kThreads)), dim3(kThreads), 0, st,
                     rowptr, col, val, n, flag);
  return hipGetLastError();
}

hipError_t launch_degree_scaling(const int64_t* rowptr, const double* val, int64_t n, double* d, double* s, int* flag,
                                 hipStream_t st) {
  hipLaunchKernelGGL(degree_kernel, dim3((unsigned)ceil_div64(n * 16, kThreads)), dim3(kThreads), 0, st, rowptr, val,
                     n, d, s, flag);
  return hipGetLastError();
}

hipError_t launch_pack_scaled(const double* x, int64_t ldx, const double* s, int64_t n, int b, double* z,
                              hipStream_t st) {
  hipLaunchKernelGGL(pack_scaled_kernel, dim3((unsigned)ceil_div64(n * b, kThreads)), dim3(kThreads), 0, st, x, ldx,
                     s, n, b, z);
  return hipGetLastError();
}

// lanes per row of the wide-block product: the smallest power of two that covers an average row in one batch, at
// most 32 (measured on the kNN workloads: 32 lanes beat 8, 16 and 64 for every block width)
static int spmm_lanes(int b, double avg_deg) {
  int lanes = b;
  while (lanes < 32 && lanes < avg_deg) lanes *= 2;
  return lanes;
}

template <int MODE>
static hipError_t launch_spmm_cols_t(const int64_t* rowptr, const int32_t* col, const double* val, const double* s,
                                     int64_t n, const double* z, int b, double* y, int64_t ldy, double avg_deg,
                                     const double* uprev, double alpha, double shift, double beta,
                                     const int32_t* longrows, int nlong, hipStream_t st, int64_t row_begin = 0) {
  const int vec_store = (ldy % 2 == 0 && reinterpret_cast<uintptr_t>(y) % 16 == 0) ? 1 : 0;
  if (!longrows) nlong = 0;
  // grid: row tiles (a multiple of kXcds), then one workgroup per long row (rounded up to kXcds)
#define SC_LAUNCH_COLS(BB, LL)                                                                                     \
  do {                                                                                                             \
    const int64_t ntiles = ceil_div64(ceil_div64(n - row_begin, kThreads / LL), kXcds) * kXcds;                    \
    const int64_t nextra = ceil_div64(nlong, kXcds) * kXcds;                                                       \
    hipLaunchKernelGGL((spmm_cols_kernel<BB, LL, MODE>), dim3((unsigned)(ntiles + nextra)), dim3(kThreads), 0, st, \
                       rowptr, col, val, s, z, y, ldy, n, vec_store, uprev, alpha, shift, beta, ntiles, longrows,  \
                       nlong, row_begin);                                                                          \
  } while (0)
  switch (b) {
    case 8:
      switch (spmm_lanes(8, avg_deg)) {
        case 8: SC_LAUNCH_COLS(8, 8); break;
        case 16: SC_LAUNCH_COLS(8, 16); break;
        default: SC_LAUNCH_COLS(8, 32); break;
      }
      break;
    case 16:
      switch (spmm_lanes(16, avg_deg)) {
        case 16: SC_LAUNCH_COLS(16, 16); break;
        default: SC_LAUNCH_COLS(16, 32); break;
      }
      break;
    case 32: SC_LAUNCH_COLS(32, 32); break;
    default: return hipErrorInvalidValue;
  }
#undef SC_LAUNCH_COLS
  return hipGetLastError();
}

hipError_t launch_spmm(const int64_t* rowptr, const int32_t* col, const double* val, const double* s, int64_t n,
                       const double* z, int b, double* y, int64_t ldy, double avg_deg, hipStream_t st) {
  switch (b) {
    case 1: return launch_spmm_nz<1>(rowptr, col, val, s, n, z, y, ldy, avg_deg, st);
    case 2: return launch_spmm_nz<2>(rowptr, col, val, s, n, z, y, ldy, avg_deg, st);
    case 4: return launch_spmm_nz<4>(rowptr, col, val, s, n, z, y, ldy, avg_deg, st);
    default:
      if (!s) return launch_spmm_cols_t<1>(rowptr, col, val, nullptr, n, z, b, y, ldy, avg_deg, nullptr, 0.0, 0.0, 0.0,
                                           nullptr, 0, st);
      return launch_spmm_cols_t<0>(rowptr, col, val, s, n, z, b, y, ldy, avg_deg, nullptr, 0.0, 0.0, 0.0, nullptr, 0, st);
  }
}

hipError_t launch_spmv_chain(const int64_t* rowptr, const int32_t* col, const double* val, const double* s, int64_t n,
                             const double* z, double* y, double* zout, double avg_deg, hipStream_t st) {
  if (avg_deg >= 6.0) return launch_spmv_tile(rowptr, col, val, s, n, z, y, 1, avg_deg, st, zout);
  // very sparse rows: the lanes-per-row kernel, then the scaling as a pass of its own
  hipError_t e = launch_spmm_nz<1>(rowptr, col, val, s, n, z, y, 1, avg_deg, st);
  if (e != hipSuccess) return e;
  return launch_pack_scaled(y, 1, s, n, 1, zout, st);
}

hipError_t launch_scale_values(const int64_t* rowptr, const int32_t* col, const double* val, const double* s,
                               double* val_out, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(scale_values_kernel, dim3((unsigned)ceil_div64(n, kThreads / 16)), dim3(kThreads), 0, st, rowptr,
                     col, val, s, val_out, n);
  return hipGetLastError();
}

hipError_t launch_spmm_vals(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, const double* x,
                            int b, double* y, int64_t ldy, double avg_deg, const int32_t* longrows, int nlong,
                            hipStream_t st) {
  return launch_spmm_cols_t<1>(rowptr, col, val, nullptr, n, x, b, y, ldy, avg_deg, nullptr, 0.0, 0.0, 0.0, longrows,
                               nlong, st);
}

hipError_t launch_spmm_vals_cheb(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n,
                                 const double* ucur, int b, const double* uprev, double* unext, double alpha,
                                 double shift, double beta, double avg_deg, const int32_t* longrows, int nlong,
                                 hipStream_t st, int64_t row_begin) {
  if (row_begin >= n) return hipSuccess;
  return launch_spmm_cols_t<2>(rowptr, col, val, nullptr, n, ucur, b, unext, b, avg_deg, uprev, alpha, shift, beta,
                               longrows, nlong, st, row_begin);
}

ProjectPlan plan_project(int64_t n, int ja, int max_partials) {
  ProjectPlan p;
  p.nwc = ja <= 64 ? 1 : (ja <= 128 ? 2 : 4);
  const int nwr = 4 / p.nwc;
  const int coltiles = (ja + 64 * p.nwc - 1) / (64 * p.nwc);
  // about 768 workgroups in total (three per compute unit), at least 16 rows per wave slice, and no
  // more partial blocks (one per workgroup and column tile group) than the reduction is meant to sum
  int64_t panels = 768 / coltiles;
  if (panels < 16) panels = 16;
  if (panels > max_partials) panels = max_partials;
  int64_t rows = ceil_div64(n, panels);
  rows = ceil_div64(rows, 16 * nwr) * 16 * nwr;
  p.rows_per_panel = (int)rows;
  p.npart = (int)ceil_div64(n, rows);
  return p;
}

hipError_t launch_project(const double* basis, int64_t n, int64_t ld, int acol0, int ja, int bcol0, int b,
                          const ProjectPlan& plan, double* part, hipStream_t st, const int* skip) {
  if (ja <= 0) return hipSuccess;
  const int panels = plan.npart;
  const dim3 grid((unsigned)panels, (unsigned)((ja + 64 * plan.nwc - 1) / (64 * plan.nwc)));
  const int vec_ok = (ld % 4 == 0 && acol0 % 4 == 0 && (reinterpret_cast<uintptr_t>(basis) % 32 == 0)) ? 1 : 0;
  // waves that share a column tile (fewer than four tiles per workgroup) add their sums through LDS; the kernel's
  // barrier needs every wave of such a workgroup to have a tile, which one tile group (ja <= 64 * nwc) guarantees
  const int nwr = 4 / plan.nwc;
  if (nwr > 1 && ja > 64 * plan.nwc) return hipErrorInvalidValue;
  const int nt = b <= 16 ? 1 : 2;
  const size_t lds = nwr > 1 ? (size_t)(nwr - 1) * plan.nwc * 16 * nt * 64 * sizeof(double) : 0;
  if (b <= 16) {
    hipLaunchKernelGGL((project_kernel<1>), grid, dim3(kThreads), lds, st, basis, n, ld, acol0, ja, bcol0, b,
                       plan.rows_per_panel, plan.nwc, vec_ok, part, skip);
  } else {
    hipLaunchKernelGGL((project_kernel<2>), grid, dim3(kThreads), lds, st, basis, n, ld, acol0, ja, bcol0, b,
                       plan.rows_per_panel, plan.nwc, vec_ok, part, skip);
  }
  return hipGetLastError();
}

hipError_t launch_reduce_partials(const double* part, int npart, int ja, int b, double* h, double* hsum,
                                  int accumulate, double* slot, int slot_row0, hipStream_t st, const int* skip) {
  if (ja <= 0) return hipSuccess;
  const int total = ja * b;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((total + kRedElems - 1) / kRedElems)), dim3(kThreads), 0,
                     st, part, npart, ja, b, h, hsum, accumulate, slot, slot_row0, skip);
  return hipGetLastError();
}

hipError_t launch_row_gemm(double* basis, int64_t n, int64_t ld, int acol0, int kdim, const double* bmat, int ldb,
                           int ncols, int mode, int ccol0, double* out, int64_t ldo, const int32_t* rowmap,
                           hipStream_t st, const int* skip) {
  if (kdim <= 0 || ncols <= 0) return hipSuccess;
  const int vec_ok = (ld % 4 == 0 && acol0 % 4 == 0 && (reinterpret_cast<uintptr_t>(basis) % 32 == 0)) ? 1 : 0;
  constexpr int MT = 2;
  const unsigned gx = (unsigned)ceil_div64(n, 4 * 16 * MT);
  const bool pipe = kdim >= 128;  // loads one trip ahead pay from a few trips on
#define SC_LAUNCH_RG(NTV, PV, GY)                                                                                  \
  hipLaunchKernelGGL((row_gemm_kernel<NTV, MT, PV>), dim3(gx, (GY)), dim3(kThreads), 0, st, basis, n, ld, acol0,   \
                     kdim, bmat, ldb, ncols, mode, ccol0, out, ldo, vec_ok, rowmap, skip)
  if (ncols <= 16) {
    if (pipe) SC_LAUNCH_RG(1, true, 1); else SC_LAUNCH_RG(1, false, 1);
  } else if (ncols <= 32) {
    if (pipe) SC_LAUNCH_RG(2, true, 1); else SC_LAUNCH_RG(2, false, 1);
  } else {
    if (mode == 0 || (mode == 3 && ncols > 64)) return hipErrorInvalidValue;
    const unsigned gy = (unsigned)((ncols + 63) / 64);
    if (pipe) SC_LAUNCH_RG(4, true, gy); else SC_LAUNCH_RG(4, false, gy);
  }
#undef SC_LAUNCH_RG
  return hipGetLastError();
}

hipError_t launch_gram_cholesky(const double* g_in, int b, double* g_out, double* rinv, double* rout,
                                const double* rprev, double abs_tol2, double rel_tol, hipStream_t st) {
#define SC_CHOL(BB)                                                                                              \
  hipLaunchKernelGGL((chol_reg_kernel<BB>), dim3(1), dim3(64), 0, st, g_in, g_out, rinv, rout, rprev, abs_tol2, \
                     rel_tol)
  switch (b) {
    case 1: SC_CHOL(1); break;
    case 2: SC_CHOL(2); break;
    case 4: SC_CHOL(4); break;
    case 8: SC_CHOL(8); break;
    case 16: SC_CHOL(16); break;
    case 32: SC_CHOL(32); break;
    default:
      hipLaunchKernelGGL(gram_cholesky_kernel, dim3(1), dim3(kCholThreads), 0, st, g_in, b, g_out, rinv, rout, rprev,
                         abs_tol2, rel_tol);
  }
#undef SC_CHOL
  return hipGetLastError();
}

// skip[0] = 1 if a second Gram-Schmidt pass is unnecessary for every column of the block, else 0.  Column t lost
// removed_t = sum_c h[c][t]^2 of its squared norm to the first pass and kept gram[t][t]; the first pass leaves an
// orthogonality error of about eps * sqrt(1 + removed / kept), which a second pass is needed for only when
// removed > ratio2 * kept.  One workgroup; fixed summation order.
constexpr int kTestThreads = 1024;  // 32 row classes per column: the coefficient block has up to m rows
__global__ __launch_bounds__(kTestThreads) void second_pass_test_kernel(const double* __restrict__ h, int ja, int b,
                                                                        const double* __restrict__ gram, double ratio2,
                                                                        int* __restrict__ skip) {
  __shared__ double sub[kTestThreads];
  __shared__ int need;
  if (threadIdx.x == 0) need = 0;
  const int t = threadIdx.x % kPartialPad, r = threadIdx.x / kPartialPad;
  double acc = 0.0;
  if (t < b)
    for (int c = r; c < ja; c += kTestThreads / kPartialPad) {
      const double v = h[(int64_t)c * kPartialPad + t];
      acc += v * v;
    }
  sub[threadIdx.x] = acc;
  __syncthreads();
  if (r == 0 && t < b) {
    double removed = 0.0;
#pragma unroll
    for (int q = 0; q < kTestThreads / kPartialPad; ++q) removed += sub[q * kPartialPad + t];
    const double kept = gram[t * kPartialPad + t];
    if (removed > ratio2 * kept) atomicOr(&need, 1);
  }
  __syncthreads();
  if (threadIdx.x == 0) skip[0] = need ? 0 : 1;
}

// Measurement aid: nothing but fp64 matrix-core instructions, eight independent accumulators per wave, no memory
// traffic inside the loop, in either form of the instruction: 16x16x4 (2,048 flops, what the contraction kernels above
// use: one operand value per lane feeds a 16 x 16 block) or 4x4x4 (four independent 4 x 4 blocks, 512 flops).  What
// this reaches is the practical ceiling of the fp64 MFMA rate on the device (the published peak assumes the highest
// clock and the better form).
template <int SHAPE>
__global__ __launch_bounds__(kThreads) void mfma_rate_kernel(double* __restrict__ sink, int iters, double a0, double b0) {
  d4 acc[8];
  double acc1[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    acc[x] = (d4){0.0, 0.0, 0.0, 0.0};
    acc1[x] = 0.0;
  }
  const double a = a0 + 1e-9 * (double)threadIdx.x, b = b0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      if constexpr (SHAPE == 16)
        acc[x] = MFMA_F64(a, b, acc[x]);
      else
        acc1[x] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc1[x], 0, 0, 0);
    }
  }
  double sum = 0.0;
#pragma unroll
  for (int x = 0; x < 8; ++x) sum += acc[x][0] + acc[x][1] + acc[x][2] + acc[x][3] + acc1[x];
  sink[(int64_t)blockIdx.x * kThreads + threadIdx.x] = sum;
}

hipError_t launch_mfma_rate(double* sink, int shape, int workgroups, int iters, hipStream_t st) {
  if (shape == 16)
    hipLaunchKernelGGL(mfma_rate_kernel<16>, dim3((unsigned)workgroups), dim3(kThreads), 0, st, sink, iters, 1.0, 1e-3);
  else if (shape == 4)
    hipLaunchKernelGGL(mfma_rate_kernel<4>, dim3((unsigned)workgroups), dim3(kThreads), 0, st, sink, iters, 1.0, 1e-3);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_second_pass_test(const double* h, int ja, int b, const double* gram, double ratio2, int* skip,
                                   hipStream_t st) {
  hipLaunchKernelGGL(second_pass_test_kernel, dim3(1), dim3(kTestThreads), 0, st, h, ja, b, gram, ratio2, skip);
  return hipGetLastError();
}

int plan_update_gram(int64_t n) {
  const int64_t ntiles = (n + 127) / 128;
  return (int)(ntiles < 1024 ? ntiles : 1024);
}

hipError_t launch_update_gram(double* basis, int64_t n, int64_t ld, int acol0, int kdim, const double* bmat, int b,
                              int ccol0, int overwrite, double* gpart, hipStream_t st, const int* skip) {
  const int vec_ok = (ld % 4 == 0 && acol0 % 4 == 0 && (reinterpret_cast<uintptr_t>(basis) % 32 == 0)) ? 1 : 0;
  const unsigned grid = (unsigned)plan_update_gram(n);
  const bool pipe = kdim >= 128;  // loads one trip ahead pay from a few trips on
#define SC_LAUNCH_UG(NTV, PV)                                                                                     \
  hipLaunchKernelGGL((update_gram_kernel<NTV, PV>), dim3(grid), dim3(kThreads), 0, st, basis, n, ld, acol0, kdim, \
                     bmat, b, ccol0, vec_ok, overwrite, gpart, skip)
  if (b <= 16) {
    if (pipe) SC_LAUNCH_UG(1, true); else SC_LAUNCH_UG(1, false);
  } else {
    if (pipe) SC_LAUNCH_UG(2, true); else SC_LAUNCH_UG(2, false);
  }
#undef SC_LAUNCH_UG
  return hipGetLastError();
}

hipError_t launch_apply_rinv(double* basis, int64_t n, int64_t ld, int col0, int b, const double* rinv, double* z,
                             const double* s, hipStream_t st) {
  hipLaunchKernelGGL(apply_rinv_kernel, dim3((unsigned)ceil_div64(n, (int64_t)(kThreads / b) * kRinvTrips)),
                     dim3(kThreads), 0, st, basis, n, ld, col0, b, rinv, z, s);
  return hipGetLastError();
}

uint64_t random_block_key(uint64_t seed, uint64_t stream_id) {
  uint64_t x = seed ^ (stream_id * 0xD1B54A32D192ED03ull);
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

hipError_t launch_random_block(double* basis, int64_t n, int64_t ld, int col0, int b, uint64_t seed,
                               uint64_t stream_id, hipStream_t st) {
  hipLaunchKernelGGL(random_block_kernel, dim3((unsigned)ceil_div64(n * b, kThreads)), dim3(kThreads), 0, st, basis, n,
                     ld, col0, b, seed, stream_id);
  return hipGetLastError();
}

hipError_t launch_sub_cols(const double* src, int64_t lds, int scol0, double* dst, int64_t ldd, int dcol0, int w,
                           int64_t n, hipStream_t st) {
  if (w <= 0 || n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sub_cols_kernel, dim3((unsigned)ceil_div64(n * w, kThreads)), dim3(kThreads), 0, st, src, lds, scol0,
                     dst, ldd, dcol0, w, n);
  return hipGetLastError();
}

hipError_t launch_set_column(double* basis, int64_t n, int64_t ld, int col, const double* v, const int32_t* rowmap,
                             hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(set_column_kernel, dim3((unsigned)ceil_div64(n, kThreads)), dim3(kThreads), 0, st, basis, n, ld, col,
                     v, rowmap);
  return hipGetLastError();
}

hipError_t launch_copy_cols(const double* src, int64_t lds, int scol0, double* dst, int64_t ldd, int dcol0, int w,
                            int64_t n, hipStream_t st) {
  if (w <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy_cols_kernel, dim3((unsigned)ceil_div64(n * w, kThreads)), dim3(kThreads), 0, st, src, lds,
                     scol0, dst, ldd, dcol0, w, n);
  return hipGetLastError();
}

hipError_t launch_gather_cols_colmajor(const double* basis, int64_t n, int64_t ld, const int32_t* pos, int ncols,
                                       double* out, const int32_t* inv, hipStream_t st) {
  if (n <= 0 || ncols <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_cols_colmajor_kernel, dim3((unsigned)ceil_div64(n, 64), (unsigned)((ncols + 63) / 64)),
                     dim3(kThreads), 0, st, basis, n, ld, pos, ncols, out, inv);
  return hipGetLastError();
}

hipError_t launch_scale_rows_colmajor(double* out, int64_t n, int k, const double* s, const int32_t* inv, hipStream_t st) {
  if (n <= 0 || k <= 0) return hipSuccess;
  hipLaunchKernelGGL(scale_rows_colmajor_kernel, dim3((unsigned)ceil_div64(n, kThreads)), dim3(kThreads), 0, st, out, n,
                     k, s, inv);
  return hipGetLastError();
}

hipError_t launch_normalize_rows_colmajor(double* out, int64_t n, int k, hipStream_t st) {
  if (n <= 0 || k <= 0) return hipSuccess;
  hipLaunchKernelGGL(normalize_rows_colmajor_kernel, dim3((unsigned)ceil_div64(n, kThreads)), dim3(kThreads), 0, st, out,
                     n, k);
  return hipGetLastError();
}

hipError_t launch_cheb_combine(const double* w, const double* ycur, const double* yprev, const double* s, double alpha,
                               double shift, double beta, double* ynext, double* znext, int64_t n, int b,
                               hipStream_t st) {
  hipLaunchKernelGGL(cheb_combine_kernel, dim3((unsigned)ceil_div64(n * b, kThreads)), dim3(kThreads), 0, st, w, ycur,
                     yprev, s, alpha, shift, beta, ynext, znext, n, b);
  return hipGetLastError();
}

}  // namespace sceig

namespace sceig {

hipError_t launch_iota(int32_t* label, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(iota_kernel, dim3((unsigned)ceil_div64(n, kThreads)), dim3(kThreads), 0, st, label, n);
  return hipGetLastError();
}

hipError_t launch_cc_round(const int64_t* rowptr, const int32_t* col, const double* val, int32_t* label, int64_t n,
                           int* changed, hipStream_t st) {
  hipLaunchKernelGGL(cc_round_kernel, dim3((unsigned)ceil_div64(n * 16, kThreads)), dim3(kThreads), 0, st, rowptr,
                     col, val, label, n, changed);
  return hipGetLastError();
}

hipError_t launch_permute_csr(const int64_t* rowptr, const int32_t* col, const double* val, const int32_t* old_of_new,
                              const int32_t* new_of_old, const int64_t* rowptr_new, int32_t* col_new, double* val_new,
                              int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(permute_csr_kernel, dim3((unsigned)ceil_div64(n * 16, kThreads)), dim3(kThreads), 0, st, rowptr,
                     col, val, old_of_new, new_of_old, rowptr_new, col_new, val_new, n);
  return hipGetLastError();
}

hipError_t launch_nullspace_fill(double* basis, int64_t n, int64_t ld, int col0, int ncols, const int32_t* comp,
                                 const double* coef, hipStream_t st) {
  if (ncols <= 0) return hipSuccess;
  hipLaunchKernelGGL(nullspace_fill_kernel, dim3((unsigned)ceil_div64(n * ncols, kThreads)), dim3(kThreads), 0, st,
                     basis, n, ld, col0, ncols, comp, coef);
  return hipGetLastError();
}

}  // namespace sceig
