// Similarity-graph construction (paper Section IV-A: the similarity measures and Algorithm 1; Algorithm 2 step 4, the
// COO to CSR conversion), device kernels.
//
// Algorithm 1 centres the data in place and gives one thread a row / an edge.  Here the data are read only: a first
// kernel stores the mean and the norm of every row (of the centred row for the cross correlation), and the edge
// kernel forms sum_t (x_it - m_i)(x_jt - m_j) directly, 16 lanes per edge with 16-byte loads, so a row of the paper's
// 90 doubles is read as a few full cache lines.  The conversion sorts (row, col) keys with rocPRIM's radix sort (a
// library primitive, the counterpart of the paper's library call) and finds the row pointers by binary search.
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
constexpr int kL = 16;  // lanes per row / per edge
inline unsigned blocks(int64_t n) { return (unsigned)((n + kT - 1) / kT); }

__device__ __forceinline__ double group_sum(double v) {
#pragma unroll
  for (int o = kL / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kL);
  return v;
}

// mean[i] = (1/d) sum_t x_it (0 when centre == 0), norm[i] = |x_i - mean[i]|_2
__global__ __launch_bounds__(kT) void row_stats_kernel(const double* __restrict__ x, int64_t ldx, int64_t n, int d,
                                                       int centre, double* __restrict__ mean,
                                                       double* __restrict__ norm) {
  const int lane = threadIdx.x % kL;
  const int64_t i = (int64_t)blockIdx.x * (kT / kL) + threadIdx.x / kL;
  if (i >= n) return;
  const double* xi = x + i * ldx;
  double m = 0.0;
  if (centre) {
    double acc = 0.0;
    for (int t = lane; t < d; t += kL) acc += xi[t];
    m = group_sum(acc) / (double)d;
  }
  double ss = 0.0;
  for (int t = lane; t < d; t += kL) {
    const double c = xi[t] - m;
    ss += c * c;
  }
  ss = group_sum(ss);
  if (lane == 0) {
    mean[i] = m;
    norm[i] = sqrt(ss);
  }
}

// measure 0 / 1: val[e] = <x_u - m_u, x_v - m_v> / (norm_u norm_v)  (m = 0 for the cosine measure)
// measure 2:     val[e] = exp(-|x_u - x_v|^2 / (2 sigma^2))
__global__ __launch_bounds__(kT) void edge_similarity_kernel(const double* __restrict__ x, int64_t ldx, int d,
                                                             const int32_t* __restrict__ eu,
                                                             const int32_t* __restrict__ ev, int64_t nedges,
                                                             int measure, double inv_two_sigma2,
                                                             const double* __restrict__ mean,
                                                             const double* __restrict__ norm, int vec_ok,
                                                             int64_t n, int* __restrict__ bad,
                                                             double* __restrict__ val) {
  const int lane = threadIdx.x % kL;
  const int64_t e = (int64_t)blockIdx.x * (kT / kL) + threadIdx.x / kL;
  if (e >= nedges) return;
  const int64_t u = eu[e], v = ev[e];
  if (u < 0 || u >= n || v < 0 || v >= n) {  // uniform over the edge's lanes; no row is touched
    if (lane == 0) {
      atomicOr(bad, 1);
      val[e] = __longlong_as_double(0x7ff8000000000000ll);
    }
    return;
  }
  const double* xu = x + u * ldx;
  const double* xv = x + v * ldx;
  double mu = 0.0, mv = 0.0;
  if (measure != 2) {
    mu = mean[u];
    mv = mean[v];
  }
  double acc = 0.0;
  int t0 = 0;
  if (vec_ok) {  // rows start 16-byte aligned: pairs of coordinates per load
    const int d2 = d / 2;
    const double2* pu = reinterpret_cast<const double2*>(xu);
    const double2* pv = reinterpret_cast<const double2*>(xv);
    for (int t = lane; t < d2; t += kL) {
      const double2 a = pu[t], b = pv[t];
      if (measure == 2) {
        const double p = a.x - b.x, q = a.y - b.y;
        acc += p * p;
        acc += q * q;
      } else {
        acc += (a.x - mu) * (b.x - mv);
        acc += (a.y - mu) * (b.y - mv);
      }
    }
    t0 = 2 * d2;
  }
  for (int t = t0 + lane; t < d; t += kL) {
    if (measure == 2) {
      const double p = xu[t] - xv[t];
      acc += p * p;
    } else {
      acc += (xu[t] - mu) * (xv[t] - mv);
    }
  }
  acc = group_sum(acc);
  if (lane == 0) val[e] = measure == 2 ? exp(-acc * inv_two_sigma2) : acc / (norm[u] * norm[v]);
}

// key[p] = row << 32 | col of output entry p, src[p] = the listed entry it copies.  Entry e gives output e; with
// symmetrize its mirror (col, row) is output nnz_in + e, or a key of all ones (sorted past the end, then dropped) when
// row == col.
__global__ __launch_bounds__(kT) void coo_keys_kernel(const int32_t* __restrict__ row, const int32_t* __restrict__ col,
                                                      int64_t nnz_in, int symmetrize, int64_t n,
                                                      uint64_t* __restrict__ key, uint32_t* __restrict__ src,
                                                      int* __restrict__ bad) {
  const int64_t e = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (e >= nnz_in) return;
  const int64_t r = row[e], c = col[e];
  if (r < 0 || r >= n || c < 0 || c >= n) {
    atomicOr(bad, 1);
    key[e] = ~0ull;
    src[e] = (uint32_t)e;
    if (symmetrize) {
      key[nnz_in + e] = ~0ull;
      src[nnz_in + e] = (uint32_t)e;
    }
    return;
  }
  key[e] = ((uint64_t)r << 32) | (uint64_t)c;
  src[e] = (uint32_t)e;
  if (symmetrize) {
    key[nnz_in + e] = r == c ? ~0ull : (((uint64_t)c << 32) | (uint64_t)r);
    src[nnz_in + e] = (uint32_t)e;
  }
}

// rowptr[i] = first sorted position whose row is >= i, i = 0 .. n (keys of all ones count as row 2^32 - 1 >= n)
__global__ __launch_bounds__(kT) void coo_rowptr_kernel(const uint64_t* __restrict__ key, int64_t total, int64_t n,
                                                        int64_t* __restrict__ rowptr) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i > n) return;
  int64_t lo = 0, hi = total;
  while (lo < hi) {
    const int64_t mid = (lo + hi) / 2;
    if ((int64_t)(key[mid] >> 32) < i) {
      lo = mid + 1;
    } else {
      hi = mid;
    }
  }
  rowptr[i] = lo;
}

__global__ __launch_bounds__(kT) void coo_emit_kernel(const uint64_t* __restrict__ key, const uint32_t* __restrict__ src,
                                                      const double* __restrict__ val, int64_t nnz_out,
                                                      int32_t* __restrict__ col_out, double* __restrict__ val_out) {
  const int64_t p = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (p >= nnz_out) return;
  col_out[p] = (int32_t)(key[p] & 0xffffffffull);
  val_out[p] = val[src[p]];
}

int key_bits(int64_t n) {
  int b = 1;
  while (b < 32 && ((int64_t)1 << b) < n) ++b;
  return b;
}

}  // namespace

hipError_t launch_row_stats(const double* x, int64_t ldx, int64_t n, int d, int centre, double* mean, double* norm,
                            hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(row_stats_kernel, dim3(blocks(n * kL)), dim3(kT), 0, st, x, ldx, n, d, centre, mean, norm);
  return hipGetLastError();
}

hipError_t launch_edge_similarity(const double* x, int64_t ldx, int d, const int32_t* eu, const int32_t* ev,
                                  int64_t nedges, int measure, double sigma, const double* mean, const double* norm,
                                  int64_t n, int* bad, double* val, hipStream_t st) {
  if (nedges <= 0) return hipSuccess;
  const int vec_ok = (ldx % 2 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0) ? 1 : 0;
  const double inv = measure == 2 ? 1.0 / (2.0 * sigma * sigma) : 0.0;
  hipLaunchKernelGGL(edge_similarity_kernel, dim3(blocks(nedges * kL)), dim3(kT), 0, st, x, ldx, d, eu, ev, nedges,
                     measure, inv, mean, norm, vec_ok, n, bad, val);
  return hipGetLastError();
}

size_t coo_to_csr_workspace(int64_t total) {
  size_t sort_bytes = 0;
  (void)rocprim::radix_sort_pairs(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                  (const uint32_t*)nullptr, (uint32_t*)nullptr, (size_t)total, 0u, 64u,
                                  (hipStream_t) nullptr);
  sort_bytes = (sort_bytes + 255) / 256 * 256;
  // temp | key[total] | key_sorted[total] | src[total] | src_sorted[total]
  return sort_bytes + (size_t)total * 24 + 1024;
}

// Entries sorted by (row, col); listed duplicates stay separate entries in listing order (the sort is stable).
// rowptr_out[n] is the number of entries emitted; col_out / val_out need room for `total` entries,
// total = nnz_in * (symmetrize ? 2 : 1) < 2^31.  bad: device int, |= 1 if an index is out of range.
hipError_t coo_to_csr(const int32_t* row, const int32_t* col, const double* val, int64_t nnz_in, int64_t n,
                      int symmetrize, void* work, size_t work_bytes, int64_t* rowptr_out, int32_t* col_out,
                      double* val_out, int* bad, hipStream_t st) {
  const int64_t total = nnz_in * (symmetrize ? 2 : 1);
  if (total <= 0 || total > INT32_MAX) return hipErrorInvalidValue;
  size_t sort_bytes = 0;
  hipError_t e = rocprim::radix_sort_pairs(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                           (const uint32_t*)nullptr, (uint32_t*)nullptr, (size_t)total, 0u, 64u, st);
  if (e != hipSuccess) return e;
  const size_t tmp = (sort_bytes + 255) / 256 * 256;
  if (work_bytes < tmp + (size_t)total * 24) return hipErrorInvalidValue;
  char* base = static_cast<char*>(work);
  uint64_t* key = reinterpret_cast<uint64_t*>(base + tmp);
  uint64_t* key_sorted = key + total;
  uint32_t* src = reinterpret_cast<uint32_t*>(key_sorted + total);
  uint32_t* src_sorted = src + total;
  hipLaunchKernelGGL(coo_keys_kernel, dim3(blocks(nnz_in)), dim3(kT), 0, st, row, col, nnz_in, symmetrize, n, key, src,
                     bad);
  size_t sb = sort_bytes;
  // all 64 bits when dropped entries (keys of all ones) may be present, else only the bits that indices use
  const int end_bit = symmetrize ? 64 : 32 + key_bits(n);
  e = rocprim::radix_sort_pairs(base, sb, key, key_sorted, src, src_sorted, (size_t)total, 0u, (unsigned)end_bit, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(coo_rowptr_kernel, dim3(blocks(n + 1)), dim3(kT), 0, st, key_sorted, total, n, rowptr_out);
  // entries past rowptr[n] are the dropped ones; emitting them too is harmless (col = 2^32 - 1 truncated) but the
  // caller's arrays hold exactly `total` slots, so emit everything and let rowptr[n] say how many count
  hipLaunchKernelGGL(coo_emit_kernel, dim3(blocks(total)), dim3(kT), 0, st, key_sorted, src_sorted, val, total, col_out,
                     val_out);
  return hipGetLastError();
}

}  // namespace sceig
