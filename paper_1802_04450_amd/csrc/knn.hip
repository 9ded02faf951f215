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
constexpr int kJU = 4;   // candidates in flight (the asm statements that pin the order name four sums)
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
        asm volatile("" : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]));  // the four sums advance together
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // the sums stay in front of the tests
#pragma unroll
    for (int u = 0; u < kJU; ++u) {
      const int64_t j = j0 + u;
      const bool pass = (j < n) & (j != i) & ((acc[u] < thr) | ((acc[u] == thr) & ((int32_t)j < thr_idx)));
      if (pass) {  // bitwise, not short-circuit: the sums must not be moved behind a test of j
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

// The same search for rows of at most 32 (padded) coordinates: the queries sit in registers, NQ per thread, and the
// candidates come through LDS in tiles of kTC rows that the workgroup copies with coalesced loads (the next tile is
// fetched into registers while the current one is used; one barrier per tile).  All lanes read the same candidate
// coordinate at the same time (an LDS broadcast), so no load of the inner loop waits on memory.  Tiles are small (16
// rows) so that four workgroups fit a compute unit beside their lists (two waves per SIMD).  What bounds the loop is
// the LDS itself: a broadcast read hands 16 bytes to each of 64 lanes, 1 KB over a 128-byte-per-cycle path, and there
// is one such read for every four subtract / multiply-add pairs.
constexpr int kTC = 16;  // candidates per tile
template <int DP, int NQ>
__global__ __launch_bounds__(kQ) void knn_tile_kernel(const double* __restrict__ xp, int64_t n, int k,
                                                      int32_t* __restrict__ idx_out, double* __restrict__ dist_out) {
  constexpr int TD2 = kTC * DP / 2;    // 16-byte elements of a tile
  constexpr int NPRE = (TD2 + kQ - 1) / kQ;
  constexpr int QW = kQ * NQ;          // queries per workgroup = columns of the lists
  extern __shared__ double lds[];
  double2* yt = reinterpret_cast<double2*>(lds);                 // [2][kTC][DP/2]
  double* bd = lds + 2 * kTC * DP;                               // [k][QW]
  int32_t* bi = reinterpret_cast<int32_t*>(bd + (size_t)k * QW); // [k][QW]
  const int tid = threadIdx.x;
  int64_t qi[NQ];       // this thread's queries: one in each block of kQ consecutive points
  int col[NQ];          // and their columns of the lists
  double q[NQ][DP];
  double thr[NQ];       // the worst of the kept candidates: (thr, thr_idx) in slot thr_slot; a dead query accepts nothing
  int32_t thr_idx[NQ];
  int thr_slot[NQ];
#pragma unroll
  for (int v = 0; v < NQ; ++v) {
    qi[v] = (int64_t)blockIdx.x * QW + v * kQ + tid;
    col[v] = v * kQ + tid;
    const bool live = qi[v] < n;
#pragma unroll
    for (int t = 0; t < DP; ++t) q[v][t] = live ? xp[qi[v] * DP + t] : 0.0;
    for (int s = 0; s < k; ++s) {
      bd[s * QW + col[v]] = INFINITY;
      bi[s * QW + col[v]] = INT32_MAX;
    }
    thr[v] = live ? INFINITY : -1.0;
    thr_idx[v] = INT32_MAX;
    thr_slot[v] = 0;
  }
  const double2* __restrict__ xp2 = reinterpret_cast<const double2*>(xp);
  const int64_t total2 = n * (DP / 2);
  const int64_t ntile = (n + kTC - 1) / kTC;
  double2 pre[NPRE];
#pragma unroll
  for (int u = 0; u < NPRE; ++u) {
    const int e = tid + u * kQ;
    if (e < TD2) yt[e] = e < total2 ? xp2[e] : double2{0.0, 0.0};
  }
  __syncthreads();
  for (int64_t tile = 0; tile < ntile; ++tile) {
    const int buf = (int)(tile & 1);
    // the next tile's rows, requested now and parked in LDS after this tile's arithmetic
#pragma unroll
    for (int u = 0; u < NPRE; ++u) {
      const int e = tid + u * kQ;
      const int64_t g = (tile + 1) * TD2 + e;
      pre[u] = (e < TD2 && g < total2) ? xp2[g] : double2{0.0, 0.0};
    }
    const double2* __restrict__ yb = yt + buf * TD2;
    // The tile is walked in pieces of kJU candidates x CH coordinates.  The LDS reads of a piece are issued at the top
    // of the piece before it (the first statements behind an asm statement, which the scheduler does not move code
    // across), so they are long back when the piece is used; the sums are pinned every two coordinates.
    constexpr int CH = NQ == 2 ? 4 : 8;       // coordinates per piece (DP is a multiple of 8)
    constexpr int NPC = DP / CH;              // pieces per candidate group
    constexpr int NG = kTC / kJU;             // candidate groups per tile
    double2 yp[2][kJU][CH / 2];
#pragma unroll
    for (int u = 0; u < kJU; ++u)
#pragma unroll
      for (int h = 0; h < CH / 2; ++h) yp[0][u][h] = yb[u * (DP / 2) + h];  // the same address in every lane
    double acc[NQ][kJU];
#pragma unroll
    for (int p = 0; p < NG * NPC; ++p) {
      const int g = p / NPC, pc = p % NPC, cur = p & 1;
      if (pc == 0) {
#pragma unroll
        for (int v = 0; v < NQ; ++v)
#pragma unroll
          for (int u = 0; u < kJU; ++u) acc[v][u] = 0.0;
      }
      if (p + 1 < NG * NPC) {  // the next piece's reads
        const int g1 = (p + 1) / NPC, pc1 = (p + 1) % NPC;
#pragma unroll
        for (int u = 0; u < kJU; ++u)
#pragma unroll
          for (int h = 0; h < CH / 2; ++h)
            yp[cur ^ 1][u][h] = yb[(g1 * kJU + u) * (DP / 2) + pc1 * (CH / 2) + h];
      }
#pragma unroll
      for (int h = 0; h < CH / 2; ++h) {
        const int t = pc * CH + 2 * h;
#pragma unroll
        for (int u = 0; u < kJU; ++u) {
#pragma unroll
          for (int v = 0; v < NQ; ++v) {
            const double d0 = q[v][t] - yp[cur][u][h].x;
            acc[v][u] = fma(d0, d0, acc[v][u]);
            const double d1 = q[v][t + 1] - yp[cur][u][h].y;
            acc[v][u] = fma(d1, d1, acc[v][u]);
          }
        }
        // all the sums advance together, two coordinates at a time: left alone, the compiler finishes one candidate's
        // chain of dependent multiply-adds before it starts the next and the loop runs at the latency of one
#pragma unroll
        for (int v = 0; v < NQ; ++v) asm volatile("" : "+v"(acc[v][0]), "+v"(acc[v][1]), "+v"(acc[v][2]), "+v"(acc[v][3]));
      }
      if (pc == NPC - 1) {
        const int c0 = g * kJU;
#pragma unroll
        for (int v = 0; v < NQ; ++v)
#pragma unroll
          for (int u = 0; u < kJU; ++u) {
            const int64_t j = tile * kTC + c0 + u;
            const double a = acc[v][u];
            // bitwise, not short-circuit: the sums above must not be moved behind a test of j
            const bool pass = (j < n) & (j != qi[v]) & ((a < thr[v]) | ((a == thr[v]) & ((int32_t)j < thr_idx[v])));
            if (pass) {
              bd[thr_slot[v] * QW + col[v]] = a;
              bi[thr_slot[v] * QW + col[v]] = (int32_t)j;
              double w = -1.0;
              int32_t wid = INT32_MAX;
              int ws = 0;
              for (int s = 0; s < k; ++s) {
                const double x = bd[s * QW + col[v]];
                const int32_t id = bi[s * QW + col[v]];
                if (x > w || (x == w && id > wid)) {
                  w = x;
                  wid = id;
                  ws = s;
                }
              }
              thr[v] = w;
              thr_idx[v] = wid;
              thr_slot[v] = ws;
            }
          }
      }
    }
    double2* yn = yt + (buf ^ 1) * TD2;
#pragma unroll
    for (int u = 0; u < NPRE; ++u) {
      const int e = tid + u * kQ;
      if (e < TD2) yn[e] = pre[u];
    }
    __syncthreads();  // every thread, dead queries included, passes here once per tile
  }
#pragma unroll
  for (int v = 0; v < NQ; ++v) {
    if (qi[v] >= n) continue;
    const int cq = col[v];
    for (int a = 0; a < k; ++a) {  // nearest first (ties: lower index first): selection sort of the k slots
      int best = a;
      double bv = bd[a * QW + cq];
      int32_t bid = bi[a * QW + cq];
      for (int s = a + 1; s < k; ++s) {
        const double x = bd[s * QW + cq];
        const int32_t id = bi[s * QW + cq];
        if (x < bv || (x == bv && id < bid)) {
          best = s;
          bv = x;
          bid = id;
        }
      }
      bd[best * QW + cq] = bd[a * QW + cq];
      bi[best * QW + cq] = bi[a * QW + cq];
      bd[a * QW + cq] = bv;
      bi[a * QW + cq] = bid;
      idx_out[qi[v] * k + a] = bid == INT32_MAX ? -1 : bid;
      dist_out[qi[v] * k + a] = sqrt(bv);
    }
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

int knn_padded_dim(int d) { return d <= 8 ? 8 : d <= 16 ? 16 : d <= 32 ? 32 : (d + kDC - 1) / kDC * kDC; }

size_t knn_search_lds_bytes(int d, int k) {
  const size_t lists = (size_t)kQ * k * (sizeof(double) + sizeof(int32_t));
  const int dp = knn_padded_dim(d);
  if (dp <= 32) return lists + 2 * (size_t)kTC * dp * sizeof(double);  // two candidate tiles
  return lists + (size_t)kQ * dp * sizeof(double);                     // the queries
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
  hipLaunchKernelGGL(pad_rows_kernel, dim3(blocks(n * dp)), dim3(kT), 0, st, x, ldx, n, d, dp, xp);
#define SC_KNN_TILE(DPV, NQV)                                                                                  \
  do {                                                                                                         \
    const size_t l = lds + (NQV - 1) * (size_t)kQ * k * 12;                                                    \
    if (l > 64 * 1024) {                                                                                       \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&knn_tile_kernel<DPV, NQV>),                       \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)l);                             \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    hipLaunchKernelGGL((knn_tile_kernel<DPV, NQV>), dim3((unsigned)((n + kQ * NQV - 1) / (kQ * NQV))), dim3(kQ), l, \
                       st, xp, n, k, idx_out, dist_out);                                                       \
  } while (0)
  // one query per thread: with two (NQ = 2) every LDS read feeds twice the arithmetic, but the lists of 256 queries
  // leave room for two workgroups per compute unit only (one wave per SIMD), and the search of 100,000 points in 32
  // dimensions took 69 ms instead of 50 ms
  if (dp == 8) {
    SC_KNN_TILE(8, 1);
  } else if (dp == 16) {
    SC_KNN_TILE(16, 1);
  } else if (dp == 32) {
    SC_KNN_TILE(32, 1);
  } else {
    if (lds > 64 * 1024) {
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&knn_search_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(knn_search_kernel, dim3((unsigned)((n + kQ - 1) / kQ)), dim3(kQ), lds, st, xp, n, dp, k,
                       idx_out, dist_out);
  }
#undef SC_KNN_TILE
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
