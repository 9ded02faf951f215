// k-nearest-neighbour similarity graph (paper Section III-A: two points are connected if either is among the k most
// similar points of the other), device kernels: exact brute-force search by Euclidean distance and the list of the
// graph's undirected edges.
//
// Search.  The distance that ranks the neighbours is the plain sum of squared coordinate differences in coordinate
// order (the |x|^2 + |y|^2 - 2xy expansion loses digits to cancellation), and equal distances are ranked by index,
// so the result is unique.  Up to 128 coordinates the expansion is still used, on the matrix cores, but only to screen
// the candidates (knn_mfma_kernel); beyond, a vector kernel computes every distance directly (knn_search_kernel: one
// thread per query, the query's coordinates in LDS, the candidates' read with wave-uniform addresses from a
// zero-padded copy, four candidates in flight).  Either way a query keeps its k best so far in LDS together with the
// worst of them; a candidate that beats the worst replaces it and the worst is found again by a scan of the k slots,
// which after the first few hundred candidates happens rarely.
#include <hip/hip_runtime.h>
#include <cstring>

#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/device/device_select.hpp>
#include <rocprim/functional.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include <cstdint>

#include "kernels.h"

typedef double d4 __attribute__((ext_vector_type(4)));
#define MFMA_F64(a, b, c) __builtin_amdgcn_mfma_f64_16x16x4f64((a), (b), (c), 0, 0, 0)

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

// xn[i] = sum_t xp[i][t]^2 in coordinate order
__global__ __launch_bounds__(kT) void row_norms_kernel(const double* __restrict__ xp, int64_t n, int dp,
                                                       double* __restrict__ xn) {
  const int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x;
  if (i >= n) return;
  double acc = 0.0;
  for (int t = 0; t < dp; ++t) acc = fma(xp[i * dp + t], xp[i * dp + t], acc);
  xn[i] = acc;
}

// The search with the cross term on the matrix cores.  |q - y|^2 = |q|^2 + |y|^2 - 2 q.y, and q.y over 64 queries x
// 64 candidates is a dense contraction: a workgroup of four waves owns 64 queries, wave w the 16 x 64 block of its 16
// queries, as 16x16x4 fp64 MFMAs with the queries' coordinates resident in registers and the candidates' loaded with
// 16-byte loads one step ahead.  The expanded form loses digits to cancellation, so it only screens: a candidate
// whose approximate squared distance lies below the query's threshold (the k-th best exact distance so far) plus a
// bound of the rounding error, kMarginUlps * 2^-53 * (|q|^2 + |y|^2), gets a bit in an LDS mask, and every kRound
// steps one thread per query walks its bits, computes the exact distance as the plain sum of squared differences in
// coordinate order and keeps the k best by (distance, index) exactly as the other kernels do.  The thresholds the
// screen uses are those of the last walk: they only ever shrink, so a lagging threshold lets more candidates
// through, never fewer; the result is the exact one.
// Error bound: both norms carry a relative error of dp * u (u = 2^-53), the dot product an absolute error of
// dp * u * |q||y| <= dp * u * (|q|^2 + |y|^2) / 2, the two final additions 2u more of the terms' size: together
// below (2 dp + 3) u (|q|^2 + |y|^2); the margin is twice that and more.
constexpr int kMq = 64;      // queries per workgroup
constexpr int kMt = 256;     // threads
constexpr int kRound = 2;    // steps of 64 candidates between two walks of the masks
template <int DP>
__global__ __launch_bounds__(kMt) __attribute__((amdgpu_waves_per_eu(DP <= 32 ? 3 : 2))) void knn_mfma_kernel(
    const double* __restrict__ xp, const double* __restrict__ xn, int64_t n, int k, int32_t* __restrict__ idx_out,
    double* __restrict__ dist_out) {
  constexpr int NS = DP / 4;            // MFMAs per 16 x 16 block
  // coordinates per piece of a step (the B operands of one piece are in flight).  Up to 32 coordinates the pieces are
  // 16 wide, which fits three waves per SIMD without spills (28 instead of 30 ms on 100,000 points of 32 coordinates:
  // three rounds of workgroups instead of four); at 128 coordinates three waves spill and lose (2.08 against 1.93 s
  // on 500,000 points), so the wider kernels keep 32-wide pieces and two waves.
  constexpr int KC = DP <= 32 ? (DP < 16 ? DP : 16) : 32;
  constexpr int NCH = DP / KC;           // pieces per step: 1, 2 or 4
  constexpr int NSC = KC / 4;            // MFMAs per block and piece
  constexpr double kMargin = (4.0 * DP + 16.0) * 1.1102230246251565e-16;
  extern __shared__ double lds[];
  double* bd = lds;                                   // [k][kMq]
  double* thrq = bd + (size_t)k * kMq;                // [kMq]      thresholds of the last walk
  unsigned long long* mask = reinterpret_cast<unsigned long long*>(thrq + kMq);  // [kRound][kMq]
  int32_t* bi = reinterpret_cast<int32_t*>(mask + kRound * kMq);                 // [k][kMq]
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, i = lane & 15, g = lane >> 4;
  const int64_t q0 = (int64_t)blockIdx.x * kMq;
  const double2* __restrict__ xp2 = reinterpret_cast<const double2*>(xp);

  // setup: lists, thresholds, masks
  for (int e = tid; e < k * kMq; e += kMt) {
    bd[e] = INFINITY;
    bi[e] = INT32_MAX;
  }
  for (int e = tid; e < kRound * kMq; e += kMt) mask[e] = 0ull;
  if (tid < kMq) thrq[tid] = q0 + tid < n ? INFINITY : -INFINITY;  // a query past the end lets nothing through
  // this lane's part of the A operand: query 16 wave + i, coordinates 8m + 2g, 8m + 2g + 1
  double a[NS];
  {
    const int64_t qrow = q0 + 16 * wave + i < n ? q0 + 16 * wave + i : n - 1;
#pragma unroll
    for (int m = 0; m < NS / 2; ++m) {
      const double2 v = xp2[(qrow * DP + 8 * m + 2 * g) / 2];
      a[2 * m] = v.x;
      a[2 * m + 1] = v.y;
    }
  }
  // the queries whose results this lane holds after an MFMA: 16 wave + 4 rr + g
  double qn[4];
  int64_t qidx[4];
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    qidx[rr] = q0 + 16 * wave + 4 * rr + g;
    qn[rr] = qidx[rr] < n ? xn[qidx[rr]] : 0.0;
  }
  // the walking lanes' state: lanes 0..15 of every wave, one of the wave's queries each.  A wave screens and walks
  // on its own: after the setup no barrier joins the four waves, so one wave's walk does not hold up the others.
  double thr = INFINITY;
  int32_t thr_idx = INT32_MAX;
  int thr_slot = 0;
  const int myql = 16 * wave + lane;  // meaningful for lane < 16
  const int64_t myq = q0 + myql;
  __syncthreads();

  const int64_t nstep = (n + 63) / 64;
  double2 b0[4][NSC / 2], b1[4][NSC / 2];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb) {
    const int64_t c = 16 * cb + i < n ? 16 * cb + i : n - 1;
#pragma unroll
    for (int m = 0; m < NSC / 2; ++m) b0[cb][m] = xp2[(c * DP + 8 * m + 2 * g) / 2];
  }
  d4 acc[4];
  double yn[4];
  // one piece (KC coordinates) of a step of 64 candidates: operands in bcur, the next piece's are fetched into bnxt
  auto do_piece = [&](double2 (&bcur)[4][NSC / 2], double2 (&bnxt)[4][NSC / 2], int64_t step, int kc)
                      __attribute__((always_inline)) {
    const int64_t c0 = step * 64;
    {  // the next piece: the next coordinates of this step, or the first of the next step.  Rows are clamped to the
       // last one: straight-line loads, masked out by the index test of the screen.
      const int kcn = kc + 1 < NCH ? kc + 1 : 0;
      const int64_t cn = kc + 1 < NCH ? c0 : c0 + 64;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        int64_t c = cn + 16 * cb + i;
        c = c < n ? c : n - 1;
#pragma unroll
        for (int m = 0; m < NSC / 2; ++m) bnxt[cb][m] = xp2[(c * DP + kcn * KC + 8 * m + 2 * g) / 2];
      }
    }
    if (kc == 0) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        acc[cb] = (d4){0.0, 0.0, 0.0, 0.0};
        const int64_t c = c0 + 16 * cb + i;
        yn[cb] = xn[c < n ? c : n - 1];  // used after the step's MFMAs
      }
    }
    // four independent accumulators between two MFMAs on the same one
#pragma unroll
    for (int m = 0; m < NSC / 2; ++m) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) acc[cb] = MFMA_F64(a[kc * NSC + 2 * m], bcur[cb][m].x, acc[cb]);
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) acc[cb] = MFMA_F64(a[kc * NSC + 2 * m + 1], bcur[cb][m].y, acc[cb]);
    }
    if (kc != NCH - 1) return;
    const int sr = (int)(step % kRound);
    // only the last step has candidates past the end, only the step with the workgroup's own rows a query's self
    const bool edge = (c0 + 64 > n) | ((c0 < q0 + kMq) & (c0 + 64 > q0));  // uniform
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int ql = 16 * wave + 4 * rr + g;
      const double tq = thrq[ql];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const double sum = qn[rr] + yn[cb];
        const double d2 = fma(-2.0, acc[cb][rr], sum);
        bool pass = d2 < fma(kMargin, sum, tq);
        if (edge) {
          const int64_t c = c0 + 16 * cb + i;
          pass = pass & (c < n) & (c != qidx[rr]);
        }
        if (pass) atomicOr(&mask[sr * kMq + ql], 1ull << (16 * cb + i));
      }
    }
    if (sr == kRound - 1 || step == nstep - 1) {  // uniform
      // the wave's own LDS operations complete in order; the fence keeps the compiler from moving them
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (lane < 16 && myq < n) {
        const int cq = myql;   // this lane's column of the per-query arrays
        const int64_t cbase = (step - sr) * 64;
        for (int st = 0; st <= sr; ++st) {
          unsigned long long mbits = mask[st * kMq + cq];
          mask[st * kMq + cq] = 0ull;
          while (mbits) {
            const int bit = __ffsll((long long)mbits) - 1;
            mbits &= mbits - 1;
            const int64_t j = cbase + st * 64 + bit;
            double ex = 0.0;
            const double2* __restrict__ qr = xp2 + myq * (DP / 2);
            const double2* __restrict__ yr = xp2 + j * (DP / 2);
#pragma unroll 8
            for (int t = 0; t < DP / 2; ++t) {  // rarely run: kept small, the registers belong to the MFMA loop
              const double2 qv = qr[t], yv = yr[t];
              const double d0 = qv.x - yv.x;
              ex = fma(d0, d0, ex);
              const double d1 = qv.y - yv.y;
              ex = fma(d1, d1, ex);
            }
            if (ex < thr || (ex == thr && (int32_t)j < thr_idx)) {
              bd[thr_slot * kMq + cq] = ex;
              bi[thr_slot * kMq + cq] = (int32_t)j;
              double w = -1.0;
              int32_t wid = INT32_MAX;
              int ws = 0;
              for (int s = 0; s < k; ++s) {
                const double x = bd[s * kMq + cq];
                const int32_t id = bi[s * kMq + cq];
                if (x > w || (x == w && id > wid)) {
                  w = x;
                  wid = id;
                  ws = s;
                }
              }
              thr = w;
              thr_idx = wid;
              thr_slot = ws;
            }
          }
        }
        thrq[cq] = thr;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  };
  if constexpr (NCH == 1) {
    for (int64_t step = 0; step < nstep; step += 2) {
      do_piece(b0, b1, step, 0);
      if (step + 1 < nstep) do_piece(b1, b0, step + 1, 0);
    }
  } else {  // an even number of pieces per step: every step starts on b0
    for (int64_t step = 0; step < nstep; ++step) {
#pragma unroll
      for (int kc = 0; kc < NCH; kc += 2) {
        do_piece(b0, b1, step, kc);
        do_piece(b1, b0, step, kc + 1);
      }
    }
  }
  if (lane >= 16 || myq >= n) return;
  const int tidq = myql;
  for (int aidx = 0; aidx < k; ++aidx) {  // nearest first (ties: lower index first): selection sort of the k slots
    int best = aidx;
    double bv = bd[aidx * kMq + tidq];
    int32_t bid = bi[aidx * kMq + tidq];
    for (int s = aidx + 1; s < k; ++s) {
      const double x = bd[s * kMq + tidq];
      const int32_t id = bi[s * kMq + tidq];
      if (x < bv || (x == bv && id < bid)) {
        best = s;
        bv = x;
        bid = id;
      }
    }
    bd[best * kMq + tidq] = bd[aidx * kMq + tidq];
    bi[best * kMq + tidq] = bi[aidx * kMq + tidq];
    bd[aidx * kMq + tidq] = bv;
    bi[aidx * kMq + tidq] = bid;
    idx_out[myq * k + aidx] = bid == INT32_MAX ? -1 : bid;
    dist_out[myq * k + aidx] = sqrt(bv);
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

int knn_padded_dim(int d) {
  return d <= 8 ? 8 : d <= 16 ? 16 : d <= 32 ? 32 : d <= 64 ? 64 : d <= 128 ? 128 : (d + kDC - 1) / kDC * kDC;
}

size_t knn_search_lds_bytes(int d, int k) {
  const int dp = knn_padded_dim(d);
  if (dp <= 128)  // distances, thresholds, masks, indices of the MFMA kernel
    return 8 * ((size_t)k * kMq + kMq + kRound * kMq) + 4 * (size_t)k * kMq;
  return (size_t)kQ * ((size_t)dp * sizeof(double) + (size_t)k * (sizeof(double) + sizeof(int32_t)));
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
  if (dp <= 128) {
    double* xn = xp + (size_t)n * dp;
    hipLaunchKernelGGL(row_norms_kernel, dim3(blocks(n)), dim3(kT), 0, st, xp, n, dp, xn);
    const size_t l = lds;
    const dim3 grid((unsigned)((n + kMq - 1) / kMq));
#define SC_KNN_MFMA(DPV)                                                                                       \
  do {                                                                                                         \
    if (l > 64 * 1024) {                                                                                       \
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&knn_mfma_kernel<DPV>),                            \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)l);                             \
      if (e != hipSuccess) return e;                                                                           \
    }                                                                                                          \
    hipLaunchKernelGGL(knn_mfma_kernel<DPV>, grid, dim3(kMt), l, st, xp, xn, n, k, idx_out, dist_out);         \
  } while (0)
    if (dp == 8) SC_KNN_MFMA(8);
    else if (dp == 16) SC_KNN_MFMA(16);
    else if (dp == 32) SC_KNN_MFMA(32);
    else if (dp == 64) SC_KNN_MFMA(64);
    else SC_KNN_MFMA(128);
#undef SC_KNN_MFMA
    return hipGetLastError();
  }
  if (lds > 64 * 1024) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&knn_search_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(knn_search_kernel, dim3((unsigned)((n + kQ - 1) / kQ)), dim3(kQ), lds, st, xp, n, dp, k, idx_out,
                     dist_out);
  return hipGetLastError();
}

size_t knn_pairs_workspace(int64_t n) {
  size_t scan_bytes = 0;
  (void)rocprim::exclusive_scan(nullptr, scan_bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (int32_t)0, (size_t)n,
                                rocprim::plus<int32_t>(), (hipStream_t) nullptr);
  return (scan_bytes + 255) / 256 * 256 + 2 * (size_t)n * sizeof(int32_t) + 256;
}

hipError_t launch_knn_union_pairs(const int32_t* idx, const double* dist, int64_t n, int k, double sigma, void* work,
                                  size_t work_bytes, int32_t* eu, int32_t* ev, double* val, int32_t* last_two,
                                  hipStream_t st) {
  if (n < 1 || k < 1 || n > INT32_MAX || n * k > INT32_MAX) return hipErrorInvalidValue;
  size_t scan_bytes = 0;
  hipError_t e = rocprim::exclusive_scan(nullptr, scan_bytes, (const int32_t*)nullptr, (int32_t*)nullptr, (int32_t)0,
                                         (size_t)n, rocprim::plus<int32_t>(), st);
  if (e != hipSuccess) return e;
  const size_t tmp = (scan_bytes + 255) / 256 * 256;
  if (work_bytes < tmp + 2 * (size_t)n * sizeof(int32_t)) return hipErrorInvalidValue;
  char* base = static_cast<char*>(work);
  int32_t* cnt = reinterpret_cast<int32_t*>(base + tmp);
  int32_t* off = cnt + n;
  hipLaunchKernelGGL(pair_count_kernel, dim3(blocks(n)), dim3(kT), 0, st, idx, n, k, cnt);
  size_t sb = scan_bytes;
  e = rocprim::exclusive_scan(base, sb, cnt, off, (int32_t)0, (size_t)n, rocprim::plus<int32_t>(), st);
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
