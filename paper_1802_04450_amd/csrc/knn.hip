// k-nearest-neighbour similarity graph (paper Section III-A: two points are connected if either is among the k most
// similar points of the other), device kernels: exact brute-force search by Euclidean distance and the list of the
// graph's undirected edges.
//
// Search.  One thread per query point, 128 queries per workgroup; every workgroup walks over all n candidate points.
// A candidate's coordinates are the same for all lanes, so they are read with wave-uniform addresses (the rows are
// first copied into a zero-padded array so that whole 64-byte pieces can be read); the query's own coordinates sit in
// LDS, one column per thread.  Four candidates are in flight per pass over the coordinates, so a coordinate of the
// query is read once for four subtract / multiply-add pairs: the loop is bound by the fp64 vector units.  The squared
// distance is the plain sum of squared differences in coordinate order (no |x|^2 + |y|^2 - 2xy expansion: the
// ranking of near neighbours must not suffer cancellation).  Each thread keeps its k best so far in LDS together with
// the worst of them; a candidate that beats the worst replaces it and the worst is found again by a scan of the k
// slots, which after the first few hundred candidates happens rarely.  Equal distances are ranked by index, so the
// result is unique.
#include <hip/hip_runtime.h>
#include <hipcub/hipcub.hpp>

#include <cstdint>

#include "kernels.h"

namespace sceig {
namespace {

constexpr int kT = 256;
constexpr int kQ = 128;  // queries per workgroup of the search
constexpr int kJU = 4;   // candidates in flight
constexpr int kDC = 8;   // coordinates per piece (rows are padded to a multiple of it)
inline unsigned blocks(int64_t n) { return (unsigned)((n + kT - 1) / kT); }

__global__ __launch_bounds__(kT) void pad_rows_kernel(const double* __restrict__ x, int64_t ldx, int64_t n, int d,
                                                      int dp, double* __restrict__ xp) {
  const int64_t e = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (e >= n * dp) return;
  const int64_t i = e / dp;
  const int t = (int)(e - i * dp);
  xp[e] = t < d ? x[i * ldx + t] : 0.0;
}

__global__ __launch_bounds__(kQ) void knn_search_kernel(const double* __restrict__ xp, int64_t n, int dp, int k,
                                                        int32_t* __restrict__ idx_out,
                                                        double* __restrict__ dist_out) {
  extern __shared__ double lds[];
  double* qs = lds;                                              // [dp][kQ]  the queries, one column per thread
  double* bd = qs + (size_t)dp * kQ;                             // [k][kQ]   squared distances of the best so far
  int32_t* bi = reinterpret_cast<int32_t*>(bd + (size_t)k * kQ); // [k][kQ]   their indices
  const int tid = threadIdx.x;
  const int64_t i = (int64_t)blockIdx.x * kQ + tid;
  const bool live = i < n;
  // every thread touches only its own column of the three arrays: no barrier anywhere in this kernel
  for (int t = 0; t < dp; ++t) qs[t * kQ + tid] = live ? xp[i * dp + t] : 0.0;
  for (int s = 0; s < k; ++s) {
    bd[s * kQ + tid] = INFINITY;
    bi[s * kQ + tid] = INT32_MAX;
  }
  // the worst of the kept candidates: (thr, thr_idx) in slot thr_slot; a dead lane accepts nothing
  double thr = live ? INFINITY : -1.0;
  int32_t thr_idx = INT32_MAX;
  int thr_slot = 0;
  for (int64_t j0 = 0; j0 < n; j0 += kJU) {
    const double* __restrict__ y[kJU];
#pragma unroll
    for (int u = 0; u < kJU; ++u) y[u] = xp + (j0 + u < n ? j0 + u : n - 1) * dp;  // uniform over the workgroup
    double acc[kJU];
#pragma unroll
    for (int u = 0; u < kJU; ++u) acc[u] = 0.0;
    for (int c = 0; c < dp; c += kDC) {
#pragma unroll
      for (int t = 0; t < kDC; ++t) {
        const double qv = qs[(c + t) * kQ + tid];
#pragma unroll
        for (int u = 0; u < kJU; ++u) {
          const double df = qv - y[u][c + t];
          acc[u] = fma(df, df, acc[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kJU; ++u) {
      const int64_t j = j0 + u;
      if (j < n && j != i && (acc[u] < thr || (acc[u] == thr && (int32_t)j < thr_idx))) {
        bd[thr_slot * kQ + tid] = acc[u];
        bi[thr_slot * kQ + tid] = (int32_t)j;
        thr = -1.0;
        for (int s = 0; s < k; ++s) {
          const double v = bd[s * kQ + tid];
          const int32_t id = bi[s * kQ + tid];
          if (v > thr || (v == thr && id > thr_idx)) {
            thr = v;
            thr_idx = id;
            thr_slot = s;
          }
        }
      }
    }
  }
  if (!live) return;
  // nearest first (ties: lower index first): selection sort of the k slots
  for (int a = 0; a < k; ++a) {
    int best = a;
    double bv = bd[a * kQ + tid];
    int32_t bid = bi[a * kQ + tid];
    for (int s = a + 1; s < k; ++s) {
      const double v = bd[s * kQ + tid];
      const int32_t id = bi[s * kQ + tid];
      if (v < bv || (v == bv && id < bid)) {
        best = s;
        bv = v;
        bid = id;
      }
    }
    bd[best * kQ + tid] = bd[a * kQ + tid];
    bi[best * kQ + tid] = bi[a * kQ + tid];
    bd[a * kQ + tid] = bv;
    bi[a * kQ + tid] = bid;
    idx_out[i * k + a] = bid == INT32_MAX ? -1 : bid;
    dist_out[i * k + a] = sqrt(bv);
  }
}

// Whether entry s of row i's list names an edge that this row emits: a valid neighbour j != i, not listed earlier in
// the same row, and either i < j or i is not in j's list (else row j emits the pair).
__device__ __forceinline__ bool emits(const int32_t* __restrict__ idx, int64_t n, int k, int64_t i, int s) {
  const int32_t j = idx[i * k + s];
  if (j < 0 || j >= n || j == i) return false;
  for (int q = 0; q < s; ++q)
    if (idx[i * k + q] == j) return false;
  if (i < j) return true;
  for (int q = 0; q < k; ++q)
    if (idx[(int64_t)j * k + q] == (int32_t)i) return false;
  return true;
}

__global__ __launch_bounds__(kT) void pair_count_kernel(const int32_t* __restrict__ idx, int64_t n, int k,
                                                        int32_t* __restrict__ cnt) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  int c = 0;
  for (int s = 0; s < k; ++s) c += emits(idx, n, k, i, s) ? 1 : 0;
  cnt[i] = c;
}

__global__ __launch_bounds__(kT) void pair_emit_kernel(const int32_t* __restrict__ idx, const double* __restrict__ dist,
                                                       int64_t n, int k, const int32_t* __restrict__ offset,
                                                       double inv_two_sigma2, int32_t* __restrict__ eu,
                                                       int32_t* __restrict__ ev, double* __restrict__ val) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  int64_t o = offset[i];
  for (int s = 0; s < k; ++s) {
    if (!emits(idx, n, k, i, s)) continue;
    const int32_t j = idx[i * k + s];
    const double dd = dist[i * k + s];
    eu[o] = (int32_t)i < j ? (int32_t)i : j;
    ev[o] = (int32_t)i < j ? j : (int32_t)i;
    val[o] = inv_two_sigma2 > 0.0 ? exp(-(dd * dd) * inv_two_sigma2) : dd;
    ++o;
  }
}

}  // namespace

int knn_padded_dim(int d) { return (d + kDC - 1) / kDC * kDC; }

size_t knn_search_lds_bytes(int d, int k) {
  return (size_t)kQ * ((size_t)knn_padded_dim(d) * sizeof(double) + (size_t)k * (sizeof(double) + sizeof(int32_t)));
}

hipError_t launch_knn_search(const double* x, int64_t ldx, int64_t n, int d, int k, double* xp, int32_t* idx_out,
                             double* dist_out, hipStream_t st) {
  if (n < 2 || d < 1 || k < 1 || k > n - 1 || n > INT32_MAX) return hipErrorInvalidValue;
  const int dp = knn_padded_dim(d);
  const size_t lds = knn_search_lds_bytes(d, k);
  int dev = 0, lds_max = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) return e;
  if (lds > (size_t)lds_max) return hipErrorInvalidValue;
  if (lds > 64 * 1024) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&knn_search_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(pad_rows_kernel, dim3(blocks(n * dp)), dim3(kT), 0, st, x, ldx, n, d, dp, xp);
  hipLaunchKernelGGL(knn_search_kernel, dim3((unsigned)((n + kQ - 1) / kQ)), dim3(kQ), lds, st, xp, n, dp, k, idx_out,
                     dist_out);
  return hipGetLastError();
}

size_t knn_pairs_workspace(int64_t n) {
  size_t scan_bytes = 0;
  (void)hipcub::DeviceScan::ExclusiveSum(nullptr, scan_bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (int)n,
                                         nullptr);
  return (scan_bytes + 255) / 256 * 256 + 2 * (size_t)n * sizeof(int32_t) + 256;
}

hipError_t launch_knn_union_pairs(const int32_t* idx, const double* dist, int64_t n, int k, double sigma, void* work,
                                  size_t work_bytes, int32_t* eu, int32_t* ev, double* val, int32_t* last_two,
                                  hipStream_t st) {
  if (n < 1 || k < 1 || n > INT32_MAX || n * k > INT32_MAX) return hipErrorInvalidValue;
  size_t scan_bytes = 0;
  hipError_t e = hipcub::DeviceScan::ExclusiveSum(nullptr, scan_bytes, (const int32_t*)nullptr, (int32_t*)nullptr,
                                                  (int)n, st);
  if (e != hipSuccess) return e;
  const size_t tmp = (scan_bytes + 255) / 256 * 256;
  if (work_bytes < tmp + 2 * (size_t)n * sizeof(int32_t)) return hipErrorInvalidValue;
  char* base = static_cast<char*>(work);
  int32_t* cnt = reinterpret_cast<int32_t*>(base + tmp);
  int32_t* off = cnt + n;
  hipLaunchKernelGGL(pair_count_kernel, dim3(blocks(n)), dim3(kT), 0, st, idx, n, k, cnt);
  size_t sb = scan_bytes;
  e = hipcub::DeviceScan::ExclusiveSum(base, sb, cnt, off, (int)n, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(pair_emit_kernel, dim3(blocks(n)), dim3(kT), 0, st, idx, dist, n, k, off,
                     sigma > 0.0 ? 1.0 / (2.0 * sigma * sigma) : 0.0, eu, ev, val);
  // the pair count = off[n-1] + cnt[n-1]: both handed back for the host to add
  e = hipMemcpyAsync(last_two, off + (n - 1), sizeof(int32_t), hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return e;
  e = hipMemcpyAsync(last_two + 1, cnt + (n - 1), sizeof(int32_t), hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

}  // namespace sceig
