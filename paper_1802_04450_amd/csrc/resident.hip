// Chebyshev start-block filter with the iterates resident in LDS.
//
// The filter applies d steps of the three-term recurrence  u+ = alpha (S u - shift u) - beta u-  to a block of b
// vectors (Algorithm 3 leaves the start vector free; the solver filters its re-injection blocks).  One launch of the
// general product kernel per step gathers, for every matrix entry, a whole operand row from the L2 caches, and the
// rate of those gathers - not HBM - bounds it.  But the similarity graphs here are block diagonal (one diagonal block
// per connected component, contiguous rows after the solver's renumbering), and a step of the recurrence on one block
// needs nothing from outside the block.  So one workgroup takes one diagonal block, or a slice of BS of its b
// columns, keeps the two iterates u and u- of that slice in LDS for all d steps and streams only the block's
// (col, val) entries; the per-entry gathers become LDS reads of 8 BS bytes, and nothing is written to memory until
// the last step.
//
//   * Work items (row0, nrows, col0, BS), built by the host from the list of diagonal blocks: BS is the widest
//     power of two <= b for which 2 * nrows * BS doubles (+ the block's row pointers) fit the LDS of a compute unit;
//     a block narrower than b in LDS terms becomes b / BS items, each re-streaming the block's entries.
//   * A workgroup has 32 lane groups of 32 lanes; group g owns the block's rows g, g + 32, g + 64, ...  Its lanes load
//     32 consecutive entries of a row at once; BS / 2 lanes cover one entry with 16-byte LDS reads (a lane carries
//     two adjacent columns) and the 64 / BS sub-groups of a lane group take the batch's entries round-robin; the
//     sub-group sums are combined by a fixed shuffle tree, so the result does not depend on timing.
//   * The entries never change between steps: the first batch of each group's first 8 rows stays in registers for
//     the whole launch (a block of up to 256 rows with rows of up to 32 entries then reads the matrix exactly once);
//     further rows are requested four at a time before any of them is used, and so are the further batches of a
//     long row, so that a memory latency is paid per four batches, not per batch.
//   * The new iterate of a row overwrites that row of u- in place (only the row's owner reads it), one workgroup
//     barrier per step, then the two buffers swap roles.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

#include <rocprim/device/device_scan.hpp>
#include <rocprim/device/device_select.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include "kernels.h"

namespace sceig {
namespace {

constexpr int kRT = 1024;           // threads per workgroup
constexpr int kRL = 32;             // lanes per row
constexpr int kRG = kRT / kRL;      // lane groups per workgroup
constexpr int kRKeep = 8;           // rows per group whose first batch stays in registers
constexpr int kRAhead = 4;          // batches requested together when streaming

__host__ __device__ inline size_t resident_lds_bytes(int nrows, int bs) {
  return ((size_t)2 * nrows * bs * sizeof(double) + (size_t)(nrows + 1) * sizeof(int32_t) + 15) / 16 * 16;
}

template <int BS>
__device__ __forceinline__ void resident_item(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col,
                                              const double* __restrict__ val, const double* __restrict__ x,
                                              double* __restrict__ y, int b, int d, double alpha_first,
                                              double alpha_rest, double shift, int row0, int nr, int col0,
                                              unsigned char* smem) {
  constexpr int CL = BS / 2;       // lanes per entry (two columns per lane)
  constexpr int NS = kRL / CL;     // entries a lane group handles per round
  static_assert(BS >= 2 && BS <= 32, "slice width");
  double* bufa = reinterpret_cast<double*>(smem);
  double* bufb = bufa + (size_t)nr * BS;
  int32_t* rpl = reinterpret_cast<int32_t*>(bufb + (size_t)nr * BS);
  const int tid = threadIdx.x;
  const int lane = tid % kRL, g = tid / kRL;
  const int tl = lane % CL, sg = lane / CL;
  const int64_t ebase = rowptr[row0];
  const int nnz_local = (int)(rowptr[row0 + nr] - ebase);

  // ---- stage: row pointers relative to the block's first entry, u = the slice of x, u- = 0
  for (int r = tid; r <= nr; r += kRT) rpl[r] = (int)(rowptr[row0 + r] - ebase);
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    bufa[idx] = x[(int64_t)(row0 + r) * b + col0 + t];
    bufb[idx] = 0.0;
  }
  __syncthreads();
  if (nnz_local <= 0) {  // nothing to multiply with (cannot happen for a graph with positive degrees)
    for (int idx = tid; idx < nr * BS; idx += kRT) {
      const int r = idx / BS, t = idx - r * BS;
      y[(int64_t)(row0 + r) * b + col0 + t] = 0.0;
    }
    return;  // uniform over the workgroup
  }
  const int32_t* cp = col + ebase;
  const double* vp = val + ebase;
  const unsigned last_row = (unsigned)(nr - 1);

  // entry `lane` of the batch that starts at local entry e (of a row ending at e1): local column and value; lanes
  // past the row's end take its last entry with the value 0 (the loads are never predicated)
  auto load_batch = [&](int e, int e1, int32_t& c, double& a) {
    int idx = e + lane;
    const bool in = idx < e1;
    idx = in ? idx : e1 - 1;
    idx = idx < 0 ? 0 : idx;
    const unsigned lc = (unsigned)(cp[idx] - row0);
    c = (int32_t)(lc < last_row ? lc : last_row);  // a column outside the block (not a diagonal block) stays in range
    const double av = vp[idx];
    a = in ? av : 0.0;
  };

  // ---- the register-resident batches: first batch of rows g, g + G, ..., g + (kRKeep-1) G
  int32_t kc[kRKeep];
  double ka[kRKeep];
#pragma unroll
  for (int k = 0; k < kRKeep; ++k) {
    int r = g + k * kRG;
    r = r < nr ? r : nr - 1;
    load_batch(rpl[r], rpl[r + 1], kc[k], ka[k]);
  }

  double* cur = bufa;
  double* prev = bufb;
  for (int step = 0; step < d; ++step) {
    const double alpha = step == 0 ? alpha_first : alpha_rest;
    const double beta = step == 0 ? 0.0 : 1.0;
    const double2* __restrict__ cur2 = reinterpret_cast<const double2*>(cur);
    double2* prev2 = reinterpret_cast<double2*>(prev);

    // sums of one batch (entry `lane` = (c, a)) into the lane's two accumulators
    auto batch_sum = [&](int32_t c, double a, int cnt, double& acc0, double& acc1) {
      const int rounds = (cnt + NS - 1) / NS;
      int r = 0;
#define SC_RES_ROUNDS(K)                                        \
  {                                                             \
    double2 zv[K];                                              \
    _Pragma("unroll") for (int u = 0; u < K; ++u) {             \
      const int32_t cu = __shfl(c, (r + u) * NS + sg, kRL);     \
      zv[u] = cur2[cu * CL + tl];                               \
    }                                                           \
    _Pragma("unroll") for (int u = 0; u < K; ++u) {             \
      const double au = __shfl(a, (r + u) * NS + sg, kRL);      \
      acc0 += au * zv[u].x;                                     \
      acc1 += au * zv[u].y;                                     \
    }                                                           \
    r += K;                                                     \
  }
      while (rounds - r >= 4) SC_RES_ROUNDS(4)
      if (rounds - r >= 2) SC_RES_ROUNDS(2)
      if (rounds - r >= 1) SC_RES_ROUNDS(1)
#undef SC_RES_ROUNDS
    };

    // one row, given its first batch: further batches eight at a time, shuffle tree, recurrence, store over u-
    auto do_row = [&](int r, int32_t c, double a) {
      const int e0 = rpl[r], e1 = rpl[r + 1];
      const int len = e1 - e0;
      double acc0 = 0.0, acc1 = 0.0;
      batch_sum(c, a, len < kRL ? len : kRL, acc0, acc1);
      for (int e = e0 + kRL; e < e1; e += kRL * kRAhead) {
        int32_t tc[kRAhead];
        double ta[kRAhead];
#pragma unroll
        for (int q = 0; q < kRAhead; ++q) {
          const int eq = e + q * kRL;
          load_batch(eq < e1 ? eq : e1 - 1, e1, tc[q], ta[q]);
        }
#pragma unroll
        for (int q = 0; q < kRAhead; ++q) {
          const int left = e1 - (e + q * kRL);
          if (left > 0) batch_sum(tc[q], ta[q], left < kRL ? left : kRL, acc0, acc1);
        }
      }
#pragma unroll
      for (int o = kRL / 2; o >= CL; o >>= 1) {
        acc0 += __shfl_xor(acc0, o, kRL);
        acc1 += __shfl_xor(acc1, o, kRL);
      }
      if (lane < CL) {
        const double2 own = cur2[r * CL + tl];
        const double2 pv = prev2[r * CL + tl];
        double2 out;
        out.x = alpha * (acc0 - shift * own.x) - beta * pv.x;
        out.y = alpha * (acc1 - shift * own.y) - beta * pv.y;
        prev2[r * CL + tl] = out;
      }
    };

#pragma unroll
    for (int k = 0; k < kRKeep; ++k) {
      const int r = g + k * kRG;
      if (r < nr) do_row(r, kc[k], ka[k]);
    }
    for (int rb = g + kRKeep * kRG; rb < nr; rb += kRAhead * kRG) {
      int32_t tc[kRAhead];
      double ta[kRAhead];
#pragma unroll
      for (int q = 0; q < kRAhead; ++q) {
        int r = rb + q * kRG;
        r = r < nr ? r : nr - 1;
        load_batch(rpl[r], rpl[r + 1], tc[q], ta[q]);
      }
#pragma unroll
      for (int q = 0; q < kRAhead; ++q) {
        const int r = rb + q * kRG;
        if (r < nr) do_row(r, tc[q], ta[q]);
      }
    }
    __syncthreads();  // every row of the new iterate is in place; nobody reads the old u- any more
    double* t = cur;
    cur = prev;
    prev = t;
  }
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    y[(int64_t)(row0 + r) * b + col0 + t] = cur[idx];
  }
}

__global__ __launch_bounds__(kRT) void cheb_resident_kernel(const int64_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ col,
                                                            const double* __restrict__ val,
                                                            const double* __restrict__ x, double* __restrict__ y, int b,
                                                            int d, double alpha_first, double alpha_rest, double shift,
                                                            const int32_t* __restrict__ items) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int32_t* it = items + 4 * (int64_t)blockIdx.x;
  const int row0 = it[0], nr = it[1], col0 = it[2], bs = it[3];  // uniform over the workgroup
  switch (bs) {
    case 2: resident_item<2>(rowptr, col, val, x, y, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, smem); break;
    case 4: resident_item<4>(rowptr, col, val, x, y, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, smem); break;
    case 8: resident_item<8>(rowptr, col, val, x, y, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, smem); break;
    case 16: resident_item<16>(rowptr, col, val, x, y, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, smem); break;
    case 32: resident_item<32>(rowptr, col, val, x, y, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, smem); break;
    default: break;
  }
}

// ---- diagonal blocks of a CSR matrix -------------------------------------------------------------------------------
// reach[i] = max(i, largest column of row i)
__global__ __launch_bounds__(256) void row_reach_kernel(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col,
                                                        int64_t n, int32_t* __restrict__ reach) {
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
  const int lane = threadIdx.x & 15;
  if (row >= n) return;
  const int64_t e1 = rowptr[row + 1];
  int32_t m = (int32_t)row;
  for (int64_t e = rowptr[row] + lane; e < e1; e += 16) m = max(m, col[e]);
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o, 16));
  if (lane == 0) reach[row] = m;
}

// flag[p] = 1 if row p starts a diagonal block: no row before it reaches column p or beyond
__global__ __launch_bounds__(256) void block_start_kernel(const int32_t* __restrict__ reach_prefix_max, int64_t n,
                                                          unsigned char* __restrict__ flag) {
  const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (p >= n) return;
  flag[p] = (p == 0 || (int64_t)reach_prefix_max[p - 1] < p) ? 1 : 0;
}

struct MaxOp {
  __host__ __device__ int32_t operator()(const int32_t& a, const int32_t& b) const { return a > b ? a : b; }
};

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

size_t resident_item_lds_bytes(int nrows, int bs) { return resident_lds_bytes(nrows, bs); }

size_t diagonal_blocks_workspace(int64_t n) {
  size_t t1 = 0, t2 = 0;
  (void)rocprim::inclusive_scan(nullptr, t1, (int32_t*)nullptr, (int32_t*)nullptr, (size_t)n, MaxOp());
  (void)rocprim::select(nullptr, t2, rocprim::counting_iterator<int32_t>(0), (unsigned char*)nullptr, (int32_t*)nullptr,
                        (int32_t*)nullptr, (size_t)n);
  return up256((size_t)n * 4) + up256((size_t)n) + up256(t1 > t2 ? t1 : t2) + 256;
}

hipError_t diagonal_blocks(const int64_t* rowptr, const int32_t* col, int64_t n, void* work, size_t work_bytes,
                           int32_t* starts, int32_t* count, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (work_bytes < diagonal_blocks_workspace(n)) return hipErrorInvalidValue;
  char* w = static_cast<char*>(work);
  int32_t* reach = reinterpret_cast<int32_t*>(w);
  unsigned char* flag = reinterpret_cast<unsigned char*>(w + up256((size_t)n * 4));
  void* temp = w + up256((size_t)n * 4) + up256((size_t)n);
  size_t temp_bytes = work_bytes - up256((size_t)n * 4) - up256((size_t)n);
  hipLaunchKernelGGL(row_reach_kernel, dim3((unsigned)((n * 16 + 255) / 256)), dim3(256), 0, st, rowptr, col, n, reach);
  hipError_t e = rocprim::inclusive_scan(temp, temp_bytes, reach, reach, (size_t)n, MaxOp(), st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(block_start_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, reach, n, flag);
  e = rocprim::select(temp, temp_bytes, rocprim::counting_iterator<int32_t>(0), flag, starts, count, (size_t)n, st);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t launch_cheb_resident(const int64_t* rowptr, const int32_t* col, const double* val, const double* x, double* y,
                                int b, int d, double alpha_first, double alpha_rest, double shift, const int32_t* items,
                                int nitems, size_t lds_bytes, hipStream_t st) {
  if (nitems <= 0 || d <= 0) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&cheb_resident_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cheb_resident_kernel, dim3((unsigned)nitems), dim3(kRT), lds_bytes, st, rowptr, col, val, x, y, b, d,
                     alpha_first, alpha_rest, shift, items);
  return hipGetLastError();
}

}  // namespace sceig
