// k-means on the rows of the eigenvector matrix (paper Section II Step 4, Section IV-C, Algorithms 4 and 5): device
// kernels.  The distance step is the paper's expanded form S = |v|^2 + |c|^2 - 2 V C^T with the product on the fp64
// matrix cores (row_gemm_kernel, kernels.hip); |v|^2 does not change the arg-min and is left out.  The centre update
// is sort based as in the paper (points ordered by label, every cluster a contiguous run), with a fixed summation
// order so that results are reproducible.  The seeding follows Algorithm 5 with the uniform numbers supplied by the
// host (a counter-based generator); a draw is one distance pass that also leaves block sums and one single-workgroup
// kernel that walks the sums level by level to the drawn point.
#include <hip/hip_runtime.h>
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/device/device_select.hpp>
#include <rocprim/functional.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include <cstdint>

#include "kernels.h"

namespace sceig {
namespace {

constexpr int kT = 256;
inline unsigned blocks(int64_t n) { return (unsigned)((n + kT - 1) / kT); }

// X[i, t] (row-major, leading dimension ldx >= d, zero padded) from the caller's points: coordinate t of point i at
// v[t * ldv + i] (column-major, the eigenvector output) or v[i * ldv + t] (row-major).  64 x 64 tiles through LDS so
// that reads and writes both run over consecutive addresses in the column-major case.
__global__ __launch_bounds__(kT) void points_to_rowmajor_kernel(const double* __restrict__ v, int64_t ldv, int colmajor,
                                                                int64_t n, int d, double* __restrict__ x,
                                                                int64_t ldx) {
  __shared__ double tile[64][65];
  const int64_t i0 = (int64_t)blockIdx.x * 64;
  const int t0 = blockIdx.y * 64;
  for (int idx = threadIdx.x; idx < 64 * 64; idx += kT) {
    // column-major source: consecutive threads walk the points; row-major source: they walk the coordinates
    const int a = idx / 64, b = idx % 64;
    const int64_t i = i0 + (colmajor ? b : a);
    const int t = t0 + (colmajor ? a : b);
    double val = 0.0;
    if (i < n && t < d) val = colmajor ? v[(int64_t)t * ldv + i] : v[i * ldv + t];
    tile[colmajor ? b : a][colmajor ? a : b] = val;  // tile[point][coordinate]
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * 64; idx += kT) {
    const int r = idx / 64, c = idx % 64;
    if (i0 + r < n && t0 + c < ldx) x[(i0 + r) * ldx + t0 + c] = tile[r][c];
  }
}

// ct[t * ldc + j] = c[j * ldx + t] (the right-hand operand of V C^T, zero padded to ldc columns and dpad rows) and
// cnorm[j] = |c_j|^2.  One workgroup per centre.
__global__ __launch_bounds__(kT) void centroid_operand_kernel(const double* __restrict__ c, int64_t ldx, int k, int d,
                                                              int dpad, double* __restrict__ ct, int64_t ldc,
                                                              double* __restrict__ cnorm) {
  __shared__ double part[kT / 64];
  const int j = blockIdx.x;
  double ss = 0.0;
  for (int t = threadIdx.x; t < dpad; t += kT) {
    const double val = t < d ? c[(int64_t)j * ldx + t] : 0.0;
    ct[(int64_t)t * ldc + j] = val;
    ss += val * val;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if (threadIdx.x % 64 == 0) part[threadIdx.x / 64] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int w = 0; w < kT / 64; ++w) tot += part[w];
    cnorm[j] = tot;
  }
  (void)k;
}

// label[i] = arg-min over j of cnorm[j] - 2 s[i, j] (the first one on ties); counts the labels that changed.
// 16 lanes per point.
__global__ __launch_bounds__(kT) void argmin_kernel(const double* __restrict__ s, int64_t lds, int64_t n, int k,
                                                    const double* __restrict__ cnorm, int32_t* __restrict__ label,
                                                    int* __restrict__ changes) {
  constexpr int L = 16;
  __shared__ int block_changes;
  if (threadIdx.x == 0) block_changes = 0;
  __syncthreads();
  const int lane = threadIdx.x % L;
  const int64_t i = (int64_t)blockIdx.x * (kT / L) + threadIdx.x / L;
  if (i < n) {
    double best = 1.79769313486231570815e308;
    int bj = 0x7fffffff;
    for (int j = lane; j < k; j += L) {
      const double val = cnorm[j] - 2.0 * s[i * lds + j];
      if (val < best) {  // j grows: an equal value later does not replace an earlier one
        best = val;
        bj = j;
      }
    }
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) {
      const double ob = __shfl_xor(best, o, L);
      const int oj = __shfl_xor(bj, o, L);
      if (ob < best || (ob == best && oj < bj)) {
        best = ob;
        bj = oj;
      }
    }
    if (lane == 0) {
      if (label[i] != bj) atomicAdd(&block_changes, 1);
      label[i] = bj;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && block_changes) atomicAdd(changes, block_changes);
}

__global__ __launch_bounds__(kT) void iota_fill_kernel(int32_t* __restrict__ a, int64_t n, int32_t value, int use_iota) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i < n) a[i] = use_iota ? (int32_t)i : value;
}

// start[c] = first position in the sorted label array with label >= c, c = 0 .. k
__global__ __launch_bounds__(kT) void cluster_starts_kernel(const int32_t* __restrict__ sorted_label, int64_t n, int k,
                                                            int32_t* __restrict__ start) {
  const int c = blockIdx.x * kT + threadIdx.x;
  if (c > k) return;
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    const int64_t mid = (lo + hi) / 2;
    if (sorted_label[mid] < c) {
      lo = mid + 1;
    } else {
      hi = mid;
    }
  }
  start[c] = (int32_t)lo;
}

// c[j, :] = mean of the points of cluster j (rows x[member[m]], start[j] <= m < start[j+1]); an empty cluster keeps
// its centre.  Workgroup (j, column tile of 64): wave w sums the members w, w+4, ... in order, the four partial sums
// are added in wave order.
__global__ __launch_bounds__(kT) void centroid_mean_kernel(const double* __restrict__ x, int64_t ldx, int d,
                                                           const int32_t* __restrict__ member,
                                                           const int32_t* __restrict__ start, double* __restrict__ c) {
  __shared__ double part[kT / 64][64];
  const int j = blockIdx.x;
  const int t = blockIdx.y * 64 + threadIdx.x % 64;
  const int w = threadIdx.x / 64;
  const int m0 = start[j], m1 = start[j + 1];
  double acc = 0.0;
  if (t < d)
    for (int m = m0 + w; m < m1; m += kT / 64) acc += x[(int64_t)member[m] * ldx + t];
  part[w][threadIdx.x % 64] = acc;
  __syncthreads();
  if (w == 0 && t < d && m1 > m0) {
    double tot = part[0][threadIdx.x];
    for (int q = 1; q < kT / 64; ++q) tot += part[q][threadIdx.x];
    c[(int64_t)j * ldx + t] = tot / (double)(m1 - m0);
  }
}

// dist2[i] = |x_i - x_c|^2 (first != 0) or min(dist2[i], |x_i - x_c|^2), c = *centre; bsum[block] = the sum of the
// block's 16 values of dist2 in point order.  16 lanes per point, 16 points per workgroup.
constexpr int kSeedPoints = kT / 16;
__global__ __launch_bounds__(kT) void seed_distance_kernel(const double* __restrict__ x, int64_t ldx, int d, int64_t n,
                                                           const int32_t* __restrict__ centre, int first,
                                                           double* __restrict__ dist2, double* __restrict__ bsum) {
  constexpr int L = 16;
  __shared__ double pts[kSeedPoints];
  const int lane = threadIdx.x % L;
  const int64_t i = (int64_t)blockIdx.x * kSeedPoints + threadIdx.x / L;
  double mine = 0.0;
  if (i < n) {  // uniform over the point's lanes
    const int64_t c = *centre;
    double acc = 0.0;
    for (int t = lane; t < d; t += L) {
      const double diff = x[i * ldx + t] - x[c * ldx + t];
      acc += diff * diff;
    }
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, L);
    mine = first ? acc : (acc < dist2[i] ? acc : dist2[i]);
    if (lane == 0) dist2[i] = mine;
  }
  if (lane == 0) pts[threadIdx.x / L] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
#pragma unroll
    for (int q = 0; q < kSeedPoints; ++q) tot += pts[q];
    bsum[blockIdx.x] = tot;
  }
}

// Inclusive prefix sums of one value per lane over the wave (fixed shuffle tree).
__device__ __forceinline__ double wave_inclusive(double v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(v, o, 64);
    if (lane >= o) v += up;
  }
  return v;
}

// The first position p in [0, count) with base + (v[0] + ... + v[p]) > r, searched by one wave in pieces of 64; *base
// receives the sum before that position.  -1 if there is none (then *base = base + the whole sum).
__device__ int wave_first_exceeding(const double* __restrict__ v, int64_t count, double r, double* base, int lane) {
  double acc = *base;
  for (int64_t p0 = 0; p0 < count; p0 += 64) {
    const double mine = p0 + lane < count ? v[p0 + lane] : 0.0;
    const double incl = wave_inclusive(mine, lane) + acc;
    const bool hit = p0 + lane < count && incl > r;
    const uint64_t mask = __ballot(hit);
    if (mask) {
      const int l = __ffsll((long long)mask) - 1;
      *base = __shfl(incl - mine, l, 64);
      return (int)p0 + l;
    }
    acc = __shfl(incl, 63, 64);
  }
  *base = acc;
  return -1;
}

// Algorithm 5's draw in one workgroup: total = sum of all dist2 (through the block sums), r = u * total, and the first
// point whose inclusive prefix sum exceeds r, found level by level: the 1024 threads each sum a contiguous run of
// block sums, their prefix sums name the run, one wave then finds the block inside the run and the point inside the
// block.  Every sum has a fixed order.  If rounding makes a level miss (the finer sums fall short of the coarser
// one) the last block / point of that level is taken; if no run qualifies (total = 0) the last point, as the
// definition says.
constexpr int kSelectThreads = 1024;
__global__ __launch_bounds__(kSelectThreads) void seed_select_kernel(const double* __restrict__ bsum, int64_t nb,
                                                                     const double* __restrict__ dist2, int64_t n, double u,
                                                                     int32_t* __restrict__ chosen) {
  __shared__ double wave_tot[kSelectThreads / 64];
  __shared__ double excl[kSelectThreads];
  __shared__ int first_run;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t chunk = (nb + kSelectThreads - 1) / kSelectThreads;
  const int64_t j0 = (int64_t)t * chunk;
  int64_t j1 = j0 + chunk;
  j1 = j1 < nb ? j1 : nb;
  double run = 0.0;
  for (int64_t j = j0; j < j1; ++j) run += bsum[j];
  const double incl_w = wave_inclusive(run, lane);
  if (lane == 63) wave_tot[wave] = incl_w;
  if (t == 0) first_run = kSelectThreads;
  __syncthreads();
  double offset = 0.0, total = 0.0;
#pragma unroll
  for (int w = 0; w < kSelectThreads / 64; ++w) {
    if (w < wave) offset += wave_tot[w];
    total += wave_tot[w];
  }
  const double incl = incl_w + offset;
  excl[t] = incl - run;
  const double r = u * total;
  if (j0 < j1 && incl > r) atomicMin(&first_run, t);
  __syncthreads();
  if (wave != 0) return;
  const int tr = first_run;
  if (tr == kSelectThreads) {  // nothing exceeds r: all distances are zero (or u * total rounded up to the total)
    if (lane == 0) *chosen = (int32_t)(n - 1);
    return;
  }
  const int64_t b0 = (int64_t)tr * chunk;
  int64_t b1 = b0 + chunk;
  b1 = b1 < nb ? b1 : nb;
  double base = excl[tr];
  bool missed = false;
  int jb = wave_first_exceeding(bsum + b0, b1 - b0, r, &base, lane);
  if (jb < 0) {  // the run's own sum exceeded r but its block sums, added up one by one, do not: take its last block
    jb = (int)(b1 - b0) - 1;
    missed = true;
  }
  const int64_t p0 = (b0 + jb) * kSeedPoints;
  int64_t p1 = p0 + kSeedPoints;
  p1 = p1 < n ? p1 : n;
  int jp = missed ? -1 : wave_first_exceeding(dist2 + p0, p1 - p0, r, &base, lane);
  if (jp < 0) jp = (int)(p1 - p0) - 1;
  if (lane == 0) *chosen = (int32_t)(p0 + jp);
}

// c[j, :] = x[index[j], :]
__global__ __launch_bounds__(kT) void gather_rows_kernel(const double* __restrict__ x, int64_t ldx,
                                                         const int32_t* __restrict__ index, int k,
                                                         double* __restrict__ c) {
  const int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (int64_t)k * ldx) return;
  const int64_t j = idx / ldx;
  c[idx] = x[(int64_t)index[j] * ldx + (idx - j * ldx)];
}

// part[block] = sum over the block's points of |x_i - c_label(i)|^2; fixed assignment of points to threads and a
// fixed tree, so the partial sums are reproducible.  Grid-stride over points, one thread per point and trip.
__global__ __launch_bounds__(kT) void objective_kernel(const double* __restrict__ x, int64_t ldx, int d, int64_t n,
                                                       const int32_t* __restrict__ label, const double* __restrict__ c,
                                                       double* __restrict__ part) {
  __shared__ double red[kT];
  double acc = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) {
    const double* xi = x + i * ldx;
    const double* cj = c + (int64_t)label[i] * ldx;
    double s2 = 0.0;
    for (int t = 0; t < d; ++t) {
      const double diff = xi[t] - cj[t];
      s2 += diff * diff;
    }
    acc += s2;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kT / 2; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

// out[i * ldo + t] = c[j * ldx + t] for the caller's row-major k x d centre array
__global__ __launch_bounds__(kT) void copy_rows_kernel(const double* __restrict__ src, int64_t lds_, double* __restrict__ dst,
                                                       int64_t ldd, int rows, int cols) {
  const int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (idx >= (int64_t)rows * cols) return;
  const int64_t r = idx / cols;
  const int t = (int)(idx - r * cols);
  dst[r * ldd + t] = src[r * lds_ + t];
}

int bits_for(int64_t n) {
  int b = 1;
  while (b < 31 && ((int64_t)1 << b) < n) ++b;
  return b;
}

}  // namespace

hipError_t launch_points_to_rowmajor(const double* v, int64_t ldv, int colmajor, int64_t n, int d, double* x, int64_t ldx,
                                     hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(points_to_rowmajor_kernel, dim3((unsigned)((n + 63) / 64), (unsigned)((ldx + 63) / 64)), dim3(kT), 0,
                     st, v, ldv, colmajor, n, d, x, ldx);
  return hipGetLastError();
}

hipError_t launch_centroid_operand(const double* c, int64_t ldx, int k, int d, int dpad, double* ct, int64_t ldc,
                                   double* cnorm, hipStream_t st) {
  hipLaunchKernelGGL(centroid_operand_kernel, dim3((unsigned)k), dim3(kT), 0, st, c, ldx, k, d, dpad, ct, ldc, cnorm);
  return hipGetLastError();
}

hipError_t launch_argmin(const double* s, int64_t lds, int64_t n, int k, const double* cnorm, int32_t* label,
                         int* changes, hipStream_t st) {
  hipLaunchKernelGGL(argmin_kernel, dim3(blocks(n * 16)), dim3(kT), 0, st, s, lds, n, k, cnorm, label, changes);
  return hipGetLastError();
}

hipError_t launch_fill_int32(int32_t* a, int64_t n, int32_t value, int use_iota, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(iota_fill_kernel, dim3(blocks(n)), dim3(kT), 0, st, a, n, value, use_iota);
  return hipGetLastError();
}

size_t kmeans_update_workspace(int64_t n) {
  size_t sort_bytes = 0;
  (void)rocprim::radix_sort_pairs(nullptr, sort_bytes, (const int32_t*)nullptr, (int32_t*)nullptr,
                                  (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, 0u, 32u, (hipStream_t) nullptr);
  sort_bytes = (sort_bytes + 255) / 256 * 256;
  // temp | ident[n] | sorted_label[n] | member[n]
  return sort_bytes + (size_t)n * 12 + 1024;
}

hipError_t launch_centroid_update(const double* x, int64_t ldx, int d, int64_t n, const int32_t* label, int k, void* work,
                                  size_t work_bytes, int32_t* start, double* c, hipStream_t st) {
  if (n <= 0 || n > INT32_MAX) return hipErrorInvalidValue;
  size_t sort_bytes = 0;
  hipError_t e = rocprim::radix_sort_pairs(nullptr, sort_bytes, (const int32_t*)nullptr, (int32_t*)nullptr,
                                           (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, 0u, 32u, st);
  if (e != hipSuccess) return e;
  const size_t tmp = (sort_bytes + 255) / 256 * 256;
  if (work_bytes < tmp + (size_t)n * 12) return hipErrorInvalidValue;
  char* base = static_cast<char*>(work);
  int32_t* ident = reinterpret_cast<int32_t*>(base + tmp);
  int32_t* sorted_label = ident + n;
  int32_t* member = sorted_label + n;
  hipLaunchKernelGGL(iota_fill_kernel, dim3(blocks(n)), dim3(kT), 0, st, ident, n, 0, 1);
  size_t sb = sort_bytes;
  e = rocprim::radix_sort_pairs(base, sb, label, sorted_label, ident, member, (size_t)n, 0u, (unsigned)bits_for(k), st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cluster_starts_kernel, dim3(blocks(k + 1)), dim3(kT), 0, st, sorted_label, n, k, start);
  hipLaunchKernelGGL(centroid_mean_kernel, dim3((unsigned)k, (unsigned)((d + 63) / 64)), dim3(kT), 0, st, x, ldx, d, member,
                     start, c);
  return hipGetLastError();
}

size_t kmeans_seed_workspace(int64_t n) {
  // dist2[n] | bsum[ceil(n / 16)]
  const size_t nb = (size_t)((n + kSeedPoints - 1) / kSeedPoints);
  return (size_t)n * 8 + nb * 8 + 1024;
}

// Algorithm 5.  u[0 .. k-1]: host array of uniform numbers in [0, 1).  chosen: device int32[k], the indices of the
// chosen points in the order they were drawn.  Two launches per draw.
hipError_t launch_kmeanspp(const double* x, int64_t ldx, int d, int64_t n, int k, const double* u, void* work,
                           size_t work_bytes, int32_t* chosen, hipStream_t st) {
  if (n <= 0 || n > INT32_MAX || k < 1) return hipErrorInvalidValue;
  const int64_t nb = (n + kSeedPoints - 1) / kSeedPoints;
  if (work_bytes < (size_t)n * 8 + (size_t)nb * 8) return hipErrorInvalidValue;
  double* dist2 = static_cast<double*>(work);
  double* bsum = dist2 + n;
  int64_t first = (int64_t)(u[0] * (double)n);
  first = first < n - 1 ? first : n - 1;
  hipLaunchKernelGGL(iota_fill_kernel, dim3(1), dim3(kT), 0, st, chosen, 1, (int32_t)first, 0);
  for (int i = 1; i < k; ++i) {
    hipLaunchKernelGGL(seed_distance_kernel, dim3((unsigned)nb), dim3(kT), 0, st, x, ldx, d, n, chosen + (i - 1),
                       i == 1 ? 1 : 0, dist2, bsum);
    hipLaunchKernelGGL(seed_select_kernel, dim3(1), dim3(kSelectThreads), 0, st, bsum, nb, dist2, n, u[i], chosen + i);
  }
  return hipGetLastError();
}

hipError_t launch_gather_rows(const double* x, int64_t ldx, const int32_t* index, int k, double* c, hipStream_t st) {
  hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks((int64_t)k * ldx)), dim3(kT), 0, st, x, ldx, index, k, c);
  return hipGetLastError();
}

int kmeans_objective_parts() { return 1024; }

hipError_t launch_objective(const double* x, int64_t ldx, int d, int64_t n, const int32_t* label, const double* c,
                            double* part, hipStream_t st) {
  hipLaunchKernelGGL(objective_kernel, dim3((unsigned)kmeans_objective_parts()), dim3(kT), 0, st, x, ldx, d, n, label, c,
                     part);
  return hipGetLastError();
}

hipError_t launch_copy_rows(const double* src, int64_t lds, double* dst, int64_t ldd, int rows, int cols, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy_rows_kernel, dim3(blocks((int64_t)rows * cols)), dim3(kT), 0, st, src, lds, dst, ldd, rows,
                     cols);
  return hipGetLastError();
}

}  // namespace sceig
