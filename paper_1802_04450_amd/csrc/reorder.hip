// Node renumbering of the setup pass, entirely on the device.
//
// Input: the component label of every node (the smallest node index of its connected component, from the label
// propagation kernels).  Output: a numbering in which every component is contiguous and, inside a component, nodes
// whose neighbourhoods share a node sit next to each other, the permuted row pointers, and the component index of
// every new row.  The paper renumbers nothing (its graphs go to cuSPARSE as they are); this pass exists for the
// gather locality of the sparse product on this machine and for the exact null space of Section IV-B's disconnected
// graphs.
//
// Order inside a component: min-hash of the closed neighbourhood.  Every node gets a pseudo-random 32-bit value; the
// key of node i is the smallest value found among i and its neighbours.  All nodes that share that "hub" receive
// the same key and become consecutive rows, and two nodes receive the same key with a probability equal to the
// Jaccard similarity of their neighbourhoods.  On kNN graphs of low-dimensional data this makes the rows of one
// tile gather from nearly the same operand rows (measured on the 3-D workload: single-vector product 1.8x faster);
// on the high-dimensional workloads it changes nothing measurable and costs one pass over the column indices.
// Three levels of it are used: h1 = the min-hash above, h2(i) = min of h1 over the closed neighbourhood (the smallest
// value within two hops), h3 likewise within three hops.  Nodes are ordered by (component, h3, h2, h1): neighbourhoods
// of one hub stay consecutive, hubs of one two-hop ball stay next to each other, and so on, which turns "somewhere in
// the component" into "within a few hundred rows" for most gathers (distinct 128-byte operand lines per 32-row tile
// on the 3-D workload: component order 771, one level 106, two 66, three 57; reverse Cuthill-McKee 64).
// The three values are re-hashed, cut to w = (64 - bits(n)) / 3 bits each and packed under the label into one 64-bit
// key: only their equality matters, and a collision merely interleaves two groups.
// On request (by_length: the solver asks for it when it will use the wide products), graphs with hubs (the longest
// row more than three average rows: kNN graphs of high-dimensional points, where the
// neighbourhoods of neighbours hardly overlap and no order helps the gathers) get the row length in place of the
// three-hop value: rows of similar length become neighbours, so the rows that share a wave of the wide products do
// the same number of trips, and the long rows of a component sit together.
// The sort is a stable LSD radix sort on that key: ties keep the original node order, so the numbering is a
// deterministic function of the graph.
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

__device__ inline uint32_t hash32(uint32_t x) {
  // a fixed bijective mixer: the ordering must not depend on anything but the graph
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// hout[i] = min over the closed neighbourhood of i of h, with h(x) = hin[x], or hash(x) when hin is null.
// 16 lanes per row.
__global__ __launch_bounds__(kT) void minhash_level_kernel(const int64_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col,
                                                           const uint32_t* __restrict__ hin, int64_t n,
                                                           uint32_t* __restrict__ hout) {
  constexpr int L = 16;
  const int lane = threadIdx.x % L;
  const int64_t row = (int64_t)blockIdx.x * (kT / L) + threadIdx.x / L;
  if (row >= n) return;  // uniform over the 16-lane group
  uint32_t m = hin ? hin[row] : hash32((uint32_t)row);
  const int64_t e1 = rowptr[row + 1];
  for (int64_t e = rowptr[row] + lane; e < e1; e += L) {
    const uint32_t c = (uint32_t)col[e];
    const uint32_t h = hin ? hin[c] : hash32(c);
    m = h < m ? h : m;
  }
#pragma unroll
  for (int o = L / 2; o > 0; o >>= 1) {
    const uint32_t other = __shfl_xor(m, o, L);
    m = other < m ? other : m;
  }
  if (lane == 0) hout[row] = m;
}

// *maxlen = the largest number of entries of a row (the slot must hold 0 on entry)
__global__ __launch_bounds__(kT) void max_row_len_kernel(const int64_t* __restrict__ rowptr, int64_t n,
                                                         int* __restrict__ maxlen) {
  int m = 0;
  for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) {
    const int len = (int)(rowptr[i + 1] - rowptr[i]);
    m = len > m ? len : m;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const int other = __shfl_xor(m, o, 64);
    m = other > m ? other : m;
  }
  if (threadIdx.x % 64 == 0 && m > 0) atomicMax(maxlen, m);
}

// csize[l] += 1 for every node with label l (the slots must hold 0 on entry): the sizes of the components, at the
// slots of their labels
__global__ __launch_bounds__(kT) void component_size_kernel(const int32_t* __restrict__ label, int64_t n,
                                                            int32_t* __restrict__ csize) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i < n) atomicAdd(&csize[label[i]], 1);
}

// key[i] = big << (3w + lb) | label << 3w | f << 2w | g(h2) << w | g(h1), g = the top w bits of a re-hash; ident[i] = i.
// big = 1 for the nodes of components with more than big_rows nodes (csize != null): those components come last.
// f = g(h3), or, if by_length is set and the graph has hubs (longest row > 3 average rows),
// 2^w - 1 - min(row length, 2^w - 1): rows of a component then come in order of decreasing length.
__global__ __launch_bounds__(kT) void pack_key_kernel(const int32_t* __restrict__ label, const uint32_t* __restrict__ h1,
                                                      const uint32_t* __restrict__ h2, const uint32_t* __restrict__ h3,
                                                      const int64_t* __restrict__ rowptr, const int* __restrict__ maxlen,
                                                      int by_length, int w, int64_t n, uint64_t* __restrict__ key,
                                                      int32_t* __restrict__ ident, const int32_t* __restrict__ csize,
                                                      int big_rows, int lb) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  const int sh = 32 - w;
  const bool hubs = by_length && (int64_t)(*maxlen) * n > 3 * rowptr[n];
  const uint64_t g1 = hash32(h1[i]) >> sh, g2 = hash32(h2[i]) >> sh;
  uint64_t f = hash32(h3[i]) >> sh;
  // components small enough for the LDS-resident filter: their rows by decreasing length too (the filter's sliced copy
  // pads the rows of a slice to its longest; locality inside such a component is of no consequence)
  const bool small_comp = csize && csize[label[i]] <= big_rows;
  if (hubs || small_comp) {
    const int64_t cap = ((int64_t)1 << w) - 1;
    const int64_t len = rowptr[i + 1] - rowptr[i];
    f = (uint64_t)(cap - (len < cap ? len : cap));
  }
  const uint64_t big = (csize && !small_comp) ? 1 : 0;
  key[i] = (big << (3 * w + lb)) | ((uint64_t)(uint32_t)label[i] << (3 * w)) | (f << (2 * w)) | (g2 << w) | g1;
  ident[i] = (int32_t)i;
}

// From the sorted order: the inverse map, the row lengths in the new order, and a 1 where a component begins.
__global__ __launch_bounds__(kT) void after_sort_kernel(const int64_t* __restrict__ rowptr,
                                                        const uint64_t* __restrict__ key_sorted,
                                                        const int32_t* __restrict__ old_of_new, int64_t n,
                                                        int label_shift, int32_t* __restrict__ new_of_old,
                                                        int64_t* __restrict__ len, int32_t* __restrict__ starts) {
  const int64_t p = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (p >= n) return;
  const int64_t old = old_of_new[p];
  new_of_old[old] = (int32_t)p;
  len[p] = rowptr[old + 1] - rowptr[old];
  starts[p] = (p == 0 || (key_sorted[p] >> label_shift) != (key_sorted[p - 1] >> label_shift)) ? 1 : 0;
}

__global__ __launch_bounds__(kT) void finish_kernel(const int64_t* __restrict__ len_scan,
                                                    const int64_t* __restrict__ len, int64_t n,
                                                    int64_t* __restrict__ rowptr_new, int32_t* comp_scan) {
  const int64_t p = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (p >= n) return;
  rowptr_new[p] = len_scan[p];
  if (p == n - 1) rowptr_new[n] = len_scan[p] + len[p];
  comp_scan[p] -= 1;  // inclusive count of component starts -> component index
}

inline unsigned blocks(int64_t n) { return (unsigned)((n + kT - 1) / kT); }

int bits_for(int64_t n) {
  int b = 1;
  while (b < 32 && ((int64_t)1 << b) < n) ++b;
  return b;
}

}  // namespace

namespace {
struct IsLongRow {
  const int64_t* rowptr;
  __device__ bool operator()(int32_t i) const { return rowptr[i + 1] - rowptr[i] > kLongRow; }
};
}  // namespace

size_t long_row_list_workspace(int64_t n) {
  size_t bytes = 0;
  rocprim::counting_iterator<int32_t> rows(0);
  (void)rocprim::select(nullptr, bytes, rows, (int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, IsLongRow{nullptr},
                        (hipStream_t) nullptr);
  return bytes + 256;
}

hipError_t long_row_list(const int64_t* rowptr, int64_t n, void* work, size_t work_bytes, int32_t* list, int32_t* count,
                         hipStream_t st) {
  if (n <= 0 || n > INT32_MAX) return hipErrorInvalidValue;
  rocprim::counting_iterator<int32_t> rows(0);
  size_t bytes = work_bytes;
  return rocprim::select(work, bytes, rows, list, count, (size_t)n, IsLongRow{rowptr}, st);
}

size_t order_by_component_workspace(int64_t n) {
  size_t sort_bytes = 0, scan64_bytes = 0, scan32_bytes = 0;
  (void)rocprim::radix_sort_pairs(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                  (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, 0u, 64u, (hipStream_t) nullptr);
  (void)rocprim::exclusive_scan(nullptr, scan64_bytes, (const int64_t*)nullptr, (int64_t*)nullptr, (int64_t)0, (size_t)n,
                                rocprim::plus<int64_t>(), (hipStream_t) nullptr);
  (void)rocprim::inclusive_scan(nullptr, scan32_bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n,
                                rocprim::plus<int32_t>(), (hipStream_t) nullptr);
  size_t tmp = sort_bytes > scan64_bytes ? sort_bytes : scan64_bytes;
  tmp = tmp > scan32_bytes ? tmp : scan32_bytes;
  tmp = (tmp + 255) / 256 * 256;
  // temp | key[n] | key_sorted[n] | len[n] | len_scan[n] | ident[n] (int32) | h1[n] h2[n] h3[n] (uint32)
  return tmp + (size_t)n * (8 + 8 + 8 + 8 + 4 + 12) + 1024;
}

hipError_t order_by_component(const int64_t* rowptr, const int32_t* col, const int32_t* label, int64_t n, int by_length,
                              int big_rows, void* work,
                              size_t work_bytes, int32_t* old_of_new, int32_t* new_of_old, int64_t* rowptr_new,
                              int32_t* comp_of_new, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n > INT32_MAX || !comp_of_new) return hipErrorInvalidValue;
  size_t sort_bytes = 0, scan64_bytes = 0, scan32_bytes = 0;
  hipError_t e = rocprim::radix_sort_pairs(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                           (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, 0u, 64u, st);
  if (e != hipSuccess) return e;
  e = rocprim::exclusive_scan(nullptr, scan64_bytes, (const int64_t*)nullptr, (int64_t*)nullptr, (int64_t)0, (size_t)n,
                              rocprim::plus<int64_t>(), st);
  if (e != hipSuccess) return e;
  e = rocprim::inclusive_scan(nullptr, scan32_bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (size_t)n,
                              rocprim::plus<int32_t>(), st);
  if (e != hipSuccess) return e;
  size_t tmp = sort_bytes > scan64_bytes ? sort_bytes : scan64_bytes;
  tmp = tmp > scan32_bytes ? tmp : scan32_bytes;
  tmp = (tmp + 255) / 256 * 256;
  if (work_bytes < tmp + (size_t)n * 48 + 64) return hipErrorInvalidValue;
  char* base = static_cast<char*>(work);
  void* temp = base;
  uint64_t* key = reinterpret_cast<uint64_t*>(base + tmp);
  uint64_t* key_sorted = key + n;
  int64_t* len = reinterpret_cast<int64_t*>(key_sorted + n);
  int64_t* len_scan = len + n;
  int32_t* ident = reinterpret_cast<int32_t*>(len_scan + n);
  uint32_t* h1 = reinterpret_cast<uint32_t*>(ident + n);
  uint32_t* h2 = h1 + n;
  uint32_t* h3 = h2 + n;

  hipLaunchKernelGGL(minhash_level_kernel, dim3(blocks(n * 16)), dim3(kT), 0, st, rowptr, col, (const uint32_t*)nullptr, n,
                     h1);
  hipLaunchKernelGGL(minhash_level_kernel, dim3(blocks(n * 16)), dim3(kT), 0, st, rowptr, col, h1, n, h2);
  hipLaunchKernelGGL(minhash_level_kernel, dim3(blocks(n * 16)), dim3(kT), 0, st, rowptr, col, h2, n, h3);
  // labels are node indices: bits_for(n) bits above three hash fields of w bits each
  const int lb = bits_for(n);
  const int w = (63 - lb) / 3 < 16 ? (63 - lb) / 3 : 16;  // one bit is kept for the large-component mark
  int32_t* csize = nullptr;
  if (big_rows > 0) {  // component sizes, in the buffer that takes the row lengths after the sort
    csize = reinterpret_cast<int32_t*>(len);
    hipError_t ec = hipMemsetAsync(csize, 0, (size_t)n * sizeof(int32_t), st);
    if (ec != hipSuccess) return ec;
    hipLaunchKernelGGL(component_size_kernel, dim3(blocks(n)), dim3(kT), 0, st, label, n, csize);
  }
  int* maxlen = reinterpret_cast<int*>(h3 + n);  // in the spare bytes at the end of the workspace
  hipError_t em = hipMemsetAsync(maxlen, 0, sizeof(int), st);
  if (em != hipSuccess) return em;
  hipLaunchKernelGGL(max_row_len_kernel, dim3((unsigned)(blocks(n) < 1024 ? blocks(n) : 1024)), dim3(kT), 0, st, rowptr, n,
                     maxlen);
  hipLaunchKernelGGL(pack_key_kernel, dim3(blocks(n)), dim3(kT), 0, st, label, h1, h2, h3, rowptr, maxlen, by_length,
                     w, n, key, ident, csize, big_rows, lb);
  size_t sb = sort_bytes;
  e = rocprim::radix_sort_pairs(temp, sb, key, key_sorted, ident, old_of_new, (size_t)n, 0u, (unsigned)(3 * w + lb + 1), st);
  if (e != hipSuccess) return e;
  int32_t* starts = ident;  // the identity values are no longer needed: the buffer takes the component-start marks
  hipLaunchKernelGGL(after_sort_kernel, dim3(blocks(n)), dim3(kT), 0, st, rowptr, key_sorted, old_of_new, n, 3 * w,
                     new_of_old, len, starts);
  size_t s64 = scan64_bytes;
  e = rocprim::exclusive_scan(temp, s64, len, len_scan, (int64_t)0, (size_t)n, rocprim::plus<int64_t>(), st);
  if (e != hipSuccess) return e;
  size_t s32 = scan32_bytes;
  e = rocprim::inclusive_scan(temp, s32, starts, comp_of_new, (size_t)n, rocprim::plus<int32_t>(), st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(finish_kernel, dim3(blocks(n)), dim3(kT), 0, st, len_scan, len, n, rowptr_new, comp_of_new);
  return hipGetLastError();
}

}  // namespace sceig
