// Chebyshev start-block filter with the iterates resident in LDS.
//
// The filter applies d steps of the three-term recurrence  u+ = alpha (S u - shift u) - beta u-  to a block of b
// vectors (Algorithm 3 leaves the start vector free; the solver filters its re-injection blocks).  One launch of the
// general product kernel per step gathers, for every matrix entry, a whole operand row from the L2 caches, and the
// rate of those gathers - not HBM - bounds it.  But the similarity graphs here are block diagonal (one diagonal block
// per connected component, contiguous rows after the solver's renumbering), and a step of the recurrence on one block
// needs nothing from outside the block.  So one workgroup takes one diagonal block (or a 16-column slice of it), keeps
// the two iterates u and u- in LDS for all d steps and the block's matrix entries in registers: after the first step
// nothing is read from memory, and nothing is written until the last.
//
//   * A lane carries 8 adjacent columns; CL = 4 lanes (32 columns) or 2 lanes (16 columns) form a lane group that
//     works on one piece of one row at a time, so a step needs no sum across lanes at all.
//   * Rows are cut into chunks of at most 8 CL entries (32 or 16) and the chunks, numbered in row order, are dealt
//     to the 1024 / CL lane groups; a group owns at most two chunks and keeps their entries - eight (column, value)
//     pairs per lane - in registers for the whole launch.  A hub row of several hundred entries is thus spread over
//     as many groups as it has chunks instead of being walked by one.  The kNN graphs' rows are ordered by length
//     inside a component, so the chunks that share a wave are equally long.
//   * One round: every lane group hands the round's entry from the lane that holds it to its other lanes with a DPP
//     quad permute (an ALU move, no LDS traffic), reads the 64 bytes of its 8 columns of that operand row from LDS
//     and does 8 multiply-adds.  A lane's 8 columns are four 16-byte pieces CL apart, so that one read instruction
//     of a lane group covers 16 CL contiguous bytes (a "segment": a quarter of the row).  A row of 8 CL doubles is a
//     whole number of LDS bank periods, so lane groups that read the same segment of different rows in the same
//     instruction hit the same banks.  Neighbouring lane groups therefore take the four segments in rotated order
//     (group w reads segment (t + w) mod 4 in its t-th read; its t-th pair of accumulators belongs to that segment
//     throughout), and the four groups of a 16-lane pass always touch four different segments.  Measured per step
//     on 2,000 blocks of 250 rows, 32 columns: 92 us with every group reading the segments in the same order, 59 us
//     with a row-dependent xor placement of the pieces (bank-conflict cycles still 49 % of the LDS-active cycles),
//     42 us with the rotation (conflict cycles below 0.2 %); the product-per-step kernel takes 166 us.
//   * The group that owns the first chunk of a row applies the recurrence with its own sum and stores the new row over
//     u- in place (only the row's owner reads it); the other chunks of a row park their sums in LDS, and after a
//     barrier the row's owner adds them in chunk order (fixed, so results are reproducible).  Blocks without hub rows
//     skip that barrier.  One more barrier ends the step and the two buffers swap roles.
//   * Work items (row0, rows, col0, CL, extra chunks) are built by the host from the diagonal blocks and their chunk
//     counts; an item's LDS need is 2 rows x 8 CL doubles for the iterates, 8 CL doubles per extra chunk, and two
//     int32 per row for the block's row pointers and chunk offsets.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <type_traits>

#include <rocprim/device/device_scan.hpp>
#include <rocprim/functional.hpp>
#include <rocprim/device/device_select.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include "kernels.h"

namespace sceig {
namespace {

constexpr int kRT = 1024;  // threads per workgroup
constexpr int kRK = 8;     // entries per lane and chunk
constexpr int kRS = 2;     // chunks per lane group

__host__ __device__ inline size_t resident_lds_bytes(int nrows, int cl, int extra) {
  const size_t bs = (size_t)8 * cl;
  return ((size_t)2 * nrows * bs * sizeof(double) + (size_t)extra * bs * sizeof(double) +
          (size_t)2 * (nrows + 1) * sizeof(int32_t) + 15) / 16 * 16;
}

// Entry idx = i * b + t of a random start block (the same numbers as random_block_kernel writes: uniform in [-1, 1)
// from the output function of splitmix64 applied to key + idx, key = mix of seed and block number made on the host).
__device__ __forceinline__ uint64_t res_mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
__device__ __forceinline__ double random_entry(uint64_t key, int64_t idx) {
  const uint64_t h = res_mix64(key + (uint64_t)idx);
  return 2.0 * ((double)(h >> 11) * (1.0 / 9007199254740992.0)) - 1.0;
}

template <int CTRL>
__device__ __forceinline__ int dpp_int(int v) {
  return __builtin_amdgcn_mov_dpp(v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ double dpp_double(double v) {
  return __hiloint2double(dpp_int<CTRL>(__double2hiint(v)), dpp_int<CTRL>(__double2loint(v)));
}
template <int CTRL>
__device__ __forceinline__ float dpp_float(float v) {
  return __int_as_float(dpp_int<CTRL>(__float_as_int(v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_value(double v) { return dpp_double<CTRL>(v); }
template <int CTRL>
__device__ __forceinline__ float dpp_value(float v) { return dpp_float<CTRL>(v); }
// two adjacent columns of an iterate, in the precision of the step
template <typename T> struct Pair;
template <> struct Pair<double> { using type = double2; };
template <> struct Pair<float> { using type = float2; };
// quad permute that gives every lane of a CL-lane group the value held by the group's lane Q
template <int CL, int Q>
struct GroupBcast {
  static constexpr int ctrl = CL == 4 ? Q * 0x55 : (Q == 0 ? 0xA0 : 0xF5);
};

template <int CL>
__device__ __forceinline__ void resident_item(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col,
                                              const double* __restrict__ val, const double* __restrict__ x,
                                              double* __restrict__ y, int64_t ldy, int b, int d, double alpha_first,
                                              double alpha_rest, double shift, int row0, int nr, int col0, int nx,
                                              unsigned char* smem, int d32, uint64_t rnd_key, int use_rnd) {
  constexpr int BS = 8 * CL;     // columns of the item
  constexpr int CH = kRK * CL;   // entries per chunk
  constexpr int G = kRT / CL;    // lane groups
  constexpr int RW = BS / 2;     // double2 per operand row
  double* bufa = reinterpret_cast<double*>(smem);
  double* bufb = bufa + (size_t)nr * BS;
  double* part = bufb + (size_t)nr * BS;
  int32_t* rpl = reinterpret_cast<int32_t*>(part + (size_t)nx * BS);
  int32_t* cst = rpl + (nr + 1);
  const int tid = threadIdx.x;
  const int q = tid % CL, g = tid / CL;
  // this lane's t-th piece (double2 index inside a row): segment (t + g) mod 4, position q inside the segment
  const int pc0 = ((g + 0) & 3) * CL + q, pc1 = ((g + 1) & 3) * CL + q, pc2 = ((g + 2) & 3) * CL + q,
            pc3 = ((g + 3) & 3) * CL + q;
  const int pcs[4] = {pc0, pc1, pc2, pc3};
  const int64_t ebase = rowptr[row0];
  const int nnz_local = (int)(rowptr[row0 + nr] - ebase);

  // ---- stage: row pointers relative to the block's first entry, chunk counts, u = the slice of x, u- = 0
  // (the first d32 steps run in single precision, on float iterates that take the first half of each buffer)
  for (int r = tid; r <= nr; r += kRT) rpl[r] = (int)(rowptr[row0 + r] - ebase);
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    // the operand, or (use_rnd, uniform) the random start block's entry made on the spot instead of read
    const int64_t gi = (int64_t)(row0 + r) * b + col0 + t;
    const double xv = use_rnd ? random_entry(rnd_key, gi) : x[gi];
    if (d32 > 0) {  // uniform
      reinterpret_cast<float*>(bufa)[idx] = (float)xv;
      reinterpret_cast<float*>(bufb)[idx] = 0.0f;
    } else {
      bufa[idx] = xv;
      bufb[idx] = 0.0;
    }
  }
  __syncthreads();
  for (int r = tid; r < nr; r += kRT) {
    const int len = rpl[r + 1] - rpl[r];
    cst[r + 1] = len > CH ? (len + CH - 1) / CH : 1;  // an empty row still is one (empty) chunk
  }
  if (tid == 0) cst[0] = 0;
  __syncthreads();
  if (tid < 64) {  // exclusive prefix sums of the chunk counts: 64 lanes, a contiguous run of rows each
    const int per = (nr + 63) / 64;
    const int lo = tid * per < nr ? tid * per : nr, hi = lo + per < nr ? lo + per : nr;
    int total = 0;
    for (int r = lo; r < hi; ++r) total += cst[r + 1];
    int incl = total;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (tid >= o) incl += up;
    }
    int run = incl - total;
    for (int r = lo; r < hi; ++r) {
      run += cst[r + 1];
      cst[r + 1] = run;
    }
  }
  __syncthreads();
  const int nv = cst[nr];  // chunks of the block; the host made sure that nv <= kRS * G and nv - nr == nx

  const int32_t* cp = col + ebase;
  const double* vp = val + ebase;
  const unsigned last_row = (unsigned)(nr - 1);

  // ---- the group's chunks: row, place among the row's chunks, entries (kept in registers for all steps)
  int32_t kc[kRS][kRK];
  double ka[kRS][kRK];
  int crow[kRS], cidx[kRS], cnum[kRS], krounds[kRS];
#pragma unroll
  for (int sl = 0; sl < kRS; ++sl) {
    const int v = g + sl * G;
    const bool valid = v < nv;
    int lo = 0, hi = nr;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cst[mid] <= (valid ? v : 0)) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int j = valid ? v - cst[r] : 0;
    const int e0 = rpl[r] + j * CH;
    int e1 = rpl[r + 1];
    e1 = e1 < e0 + CH ? e1 : e0 + CH;
    if (!valid) e1 = e0;
    crow[sl] = valid ? r : -1;
    cidx[sl] = j;
    cnum[sl] = cst[r + 1] - cst[r];
#pragma unroll
    for (int k = 0; k < kRK; ++k) {
      int idx = e0 + k * CL + q;
      const bool in = idx < e1;
      idx = in ? idx : (nnz_local > 0 ? (e1 > 0 ? e1 - 1 : 0) : 0);
      unsigned lc = 0;
      double av = 0.0;
      if (nnz_local > 0) {  // uniform over the workgroup
        lc = (unsigned)(cp[idx] - row0);
        av = vp[idx];
      }
      kc[sl][k] = (int32_t)(lc < last_row ? lc : last_row);  // a column outside the block stays inside LDS
      ka[sl][k] = in ? av : 0.0;
    }
    // rounds of this slot that any lane of the wave needs (uniform over the wave)
    int need = (e1 - e0 + CL - 1) / CL;
    if (valid && need < 1) need = 1;  // an empty row still gets its recurrence update
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const int other = __shfl_xor(need, o, 64);
      need = need > other ? need : other;
    }
    krounds[sl] = __builtin_amdgcn_readfirstlane(need);
  }

  // The steps [s0, s1) of the recurrence in the precision of `tag` (double or float), on iterates of that type in
  // the two buffers (their first halves for float); returns the buffer that holds the last iterate.
  float kaf[kRS][kRK];  // the entries once more in single precision
#pragma unroll
  for (int sl = 0; sl < kRS; ++sl)
#pragma unroll
    for (int k = 0; k < kRK; ++k) kaf[sl][k] = (float)ka[sl][k];
  // NE = columns per LDS read of a lane (its 8 columns are 8 / NE pieces, CL pieces apart): 2 in double precision
  // (16-byte reads, four pieces, as described at the top), 4 in single precision (16-byte reads again, two pieces).
  auto run_steps = [&](auto tag, auto ne_tag, int s0, int s1, void* bcur, void* bprev) __attribute__((always_inline)) -> void* {
  using T = decltype(tag);
  constexpr int NE = decltype(ne_tag)::value;
  constexpr int NP = 8 / NE;      // pieces per lane
  constexpr int RWv = BS / NE;    // pieces per operand row
  typedef T TV __attribute__((ext_vector_type(NE)));
  T* cur = static_cast<T*>(bcur);
  T* prev = static_cast<T*>(bprev);
  T* partt = reinterpret_cast<T*>(part);
  // this lane's t-th piece: segment (t + g) mod NP, position q inside the segment
  int pv[NP];
#pragma unroll
  for (int t = 0; t < NP; ++t) pv[t] = ((g + t) & (NP - 1)) * CL + q;
  for (int step = s0; step < s1; ++step) {
    const T alpha = (T)(step == 0 ? alpha_first : alpha_rest);
    const T beta = step == 0 ? (T)0 : (T)1;
    const T shiftt = (T)shift;
    const TV* __restrict__ curv = reinterpret_cast<const TV*>(cur);
    TV* prevv = reinterpret_cast<TV*>(prev);
#pragma unroll
    for (int sl = 0; sl < kRS; ++sl) {
      if (krounds[sl] == 0) continue;  // no lane of this wave has a chunk in this slot
      T acc[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[t] = (T)0;
#define SC_RES_ENTRY(K, Q)                                                                   \
  if constexpr (Q < CL) {                                                                    \
    const int cb = dpp_int<GroupBcast<CL, Q>::ctrl>(kc[sl][K]);                              \
    T av_;                                                                                   \
    if constexpr (sizeof(T) == 4) av_ = (T)kaf[sl][K]; else av_ = (T)ka[sl][K];              \
    const T ab = dpp_value<GroupBcast<CL, Q>::ctrl>(av_);                                    \
    const TV* zp = curv + cb * RWv;                                                          \
    TV z_[NP];                                                                               \
    _Pragma("unroll") for (int t = 0; t < NP; ++t) z_[t] = zp[pv[t]];                        \
    _Pragma("unroll") for (int t = 0; t < NP; ++t)                                           \
      _Pragma("unroll") for (int e = 0; e < NE; ++e) acc[NE * t + e] += ab * z_[t][e];       \
  }
#define SC_RES_ROUND(K)               \
  if (K < krounds[sl]) {              \
    SC_RES_ENTRY(K, 0)                \
    SC_RES_ENTRY(K, 1)                \
    SC_RES_ENTRY(K, 2)                \
    SC_RES_ENTRY(K, 3)                \
  }
      SC_RES_ROUND(0)
      SC_RES_ROUND(1)
      SC_RES_ROUND(2)
      SC_RES_ROUND(3)
      SC_RES_ROUND(4)
      SC_RES_ROUND(5)
      SC_RES_ROUND(6)
      SC_RES_ROUND(7)
#undef SC_RES_ROUND
#undef SC_RES_ENTRY
      const int r = crow[sl];
      if (r >= 0) {
        if (cidx[sl] == 0) {  // first chunk of its row: the recurrence with this chunk's sum, stored over u-
          const TV* own = curv + r * RWv;
          TV* out = prevv + r * RWv;
#pragma unroll
          for (int t = 0; t < NP; ++t) {
            const int at = pv[t];
            const TV o = own[at], pw = out[at];
            TV w;
#pragma unroll
            for (int e = 0; e < NE; ++e) w[e] = alpha * (acc[NE * t + e] - shiftt * o[e]) - beta * pw[e];
            out[at] = w;
          }
        } else {  // a further chunk: its sum waits in LDS for the row's owner
          TV* out = reinterpret_cast<TV*>(partt) + (size_t)(g + sl * G - r - 1) * RWv;
#pragma unroll
          for (int t = 0; t < NP; ++t) {
            TV w;
#pragma unroll
            for (int e = 0; e < NE; ++e) w[e] = acc[NE * t + e];
            out[pv[t]] = w;
          }
        }
      }
    }
    if (nx > 0) {  // uniform over the workgroup
      __syncthreads();
#pragma unroll
      for (int sl = 0; sl < kRS; ++sl) {
        const int r = crow[sl];
        if (r >= 0 && cidx[sl] == 0 && cnum[sl] > 1) {
          // the row's further chunks are chunks cst[r] + 1 ... of the block; chunk v parks at slot v - row(v) - 1
          const TV* src = reinterpret_cast<const TV*>(partt) + (size_t)(g + sl * G - r) * RWv;
          TV sum[NP];
#pragma unroll
          for (int t = 0; t < NP; ++t) sum[t] = src[pv[t]];
          for (int j = 2; j < cnum[sl]; ++j) {
            const TV* more = src + (size_t)(j - 1) * RWv;
#pragma unroll
            for (int t = 0; t < NP; ++t) sum[t] += more[pv[t]];
          }
          TV* out = prevv + r * RWv;
#pragma unroll
          for (int t = 0; t < NP; ++t) {
            const int at = pv[t];
            TV w = out[at];
            w += alpha * sum[t];
            out[at] = w;
          }
        }
      }
    }
    __syncthreads();  // every row of the new iterate is in place; nobody reads the old u- any more
    T* t = cur;
    cur = prev;
    prev = t;
  }
  return cur;
  };
  using Two = std::integral_constant<int, 2>;
  using Four = std::integral_constant<int, 4>;
  double* cur = bufa;
  if (d32 > 0) {
    // Single-precision steps first.  What their rounding adds to an iterate has components along every eigenvector,
    // and the steps that follow damp the unwanted ones like everything else below the interval's end: by the last six
    // double-precision steps they are back below what double precision leaves (measured on the first-step residuals:
    // no difference from six such steps on, a factor 5 at four).
    const bool in_b = run_steps(0.0f, Four{}, 0, d32, bufa, bufb) == static_cast<void*>(bufb);
    // both iterates from float to double, each inside its own buffer: everything is read before anything is written
    constexpr int PER = 10;  // nr * BS <= 10,240 (two double iterates fit the LDS)
    float ta[PER], tb[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int idx = tid + u * kRT;
      ta[u] = idx < nr * BS ? reinterpret_cast<const float*>(bufa)[idx] : 0.0f;
      tb[u] = idx < nr * BS ? reinterpret_cast<const float*>(bufb)[idx] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int idx = tid + u * kRT;
      if (idx < nr * BS) {
        bufa[idx] = (double)ta[u];
        bufb[idx] = (double)tb[u];
      }
    }
    __syncthreads();
    cur = static_cast<double*>(run_steps(0.0, Two{}, d32, d, in_b ? bufb : bufa, in_b ? bufa : bufb));
  } else {
    cur = static_cast<double*>(run_steps(0.0, Two{}, 0, d, bufa, bufb));
  }
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    y[(int64_t)(row0 + r) * ldy + col0 + t] = cur[idx];
  }
}

// The sliced form, for diagonal blocks whose entries do not fit the registers (up to about 1,250 rows): items of 8
// columns, the iterates in LDS as above, the entries read again in every step - from a copy of the block made for
// that (build_sliced_copy below): the block's rows in slices of 64, the k-th entries of a slice's rows next to each
// other, rows padded to the slice's longest with zero entries, columns as 16-bit indices inside the block.  A wave
// takes a slice, a lane a row: a round is one coalesced read of 64 (column, value) pairs, a 64-byte read of an operand
// row from LDS per lane (the four 16-byte pieces in an order rotated by the lane index, which spreads the banks) and 8
// multiply-adds; the row's sum never leaves the lane, so there are no partial sums to exchange.  The solver's
// renumbering orders the rows of a component by length, which keeps the padding of kNN graphs at a few per cent; a
// matrix whose padding exceeds a half is left to the product-per-step kernel by the planner.
constexpr int kSliceRows = 64;
constexpr int kSliceGroup = 8;  // rounds per register buffer of entries
constexpr int kSliceOwn = 2;    // slices a wave may own: items of up to 16 * 2 * 64 = 2,048 rows

__device__ __forceinline__ void resident_item_sliced(const uint16_t* __restrict__ scol, const double* __restrict__ sval,
                                                     const int64_t* __restrict__ slice_base,
                                                     const int32_t* __restrict__ slice_len,
                                                     const double* __restrict__ x, double* __restrict__ y, int64_t ldy, int b,
                                                     int d, double alpha_first, double alpha_rest, double shift,
                                                     int row0, int nr, int col0, int slice0, unsigned char* smem,
                                                     uint64_t rnd_key, int use_rnd) {
  constexpr int BS = 8;  // columns of the item
  constexpr int RW = BS / 2;
  double* bufa = reinterpret_cast<double*>(smem);
  double* bufb = bufa + (size_t)nr * BS;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int pc0 = (lane + 0) & 3, pc1 = (lane + 1) & 3, pc2 = (lane + 2) & 3, pc3 = (lane + 3) & 3;
  const int pcs[4] = {pc0, pc1, pc2, pc3};
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    const int64_t gi = (int64_t)(row0 + r) * b + col0 + t;
    bufa[idx] = use_rnd ? random_entry(rnd_key, gi) : x[gi];
    bufb[idx] = 0.0;
  }
  __syncthreads();
  const int nsl = (nr + kSliceRows - 1) / kSliceRows;
  // the wave's slices (wave, wave + 16, ...: at most kSliceOwn, which the planner guarantees): where their entries
  // start and how many rounds they take, fetched once
  const uint16_t* cps[kSliceOwn];
  const double* vps[kSliceOwn];
  int lens[kSliceOwn];
  int nown = 0;
#pragma unroll
  for (int j = 0; j < kSliceOwn; ++j) {
    const int sl = wave + j * (kRT / 64);
    const bool have = sl < nsl;
    const int64_t base = have ? slice_base[slice0 + sl] : 0;
    lens[j] = have ? __builtin_amdgcn_readfirstlane(slice_len[slice0 + sl]) : 0;
    cps[j] = scol + base + lane;
    vps[j] = sval + base + lane;
    nown += have ? 1 : 0;
  }
  // Rounds in groups of kSliceGroup, two register buffers: while one group is multiplied the entries of the next
  // are on their way, and the first group of the slice the wave turns to next (in this step or the one after) is
  // requested before the recurrence update and the step's barrier.  Whole groups run without a branch, so the LDS
  // reads of a round are issued ahead of the multiply-adds of the round before.  Requests past a slice's end read
  // the next slice's entries (the copy ends with room for the last slice's) and are not multiplied.
  int ca[kSliceGroup], cb[kSliceGroup];
  double aa[kSliceGroup], ab[kSliceGroup];
  auto load_group = [&](int (&c)[kSliceGroup], double (&a)[kSliceGroup], const uint16_t* cp, const double* vp, int k0)
                        __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < kSliceGroup; ++u) {
      c[u] = cp[(int64_t)(k0 + u) * kSliceRows];
      a[u] = vp[(int64_t)(k0 + u) * kSliceRows];
    }
  };
  if (nown > 0) load_group(ca, aa, cps[0], vps[0], 0);
  double* cur = bufa;
  double* prev = bufb;
  for (int step = 0; step < d; ++step) {
    const double alpha = step == 0 ? alpha_first : alpha_rest;
    const double beta = step == 0 ? 0.0 : 1.0;
    const double2* __restrict__ cur2 = reinterpret_cast<const double2*>(cur);
    double2* prev2 = reinterpret_cast<double2*>(prev);
#pragma unroll
    for (int j = 0; j < kSliceOwn; ++j) {
      if (j >= nown) break;  // uniform over the wave
      const int sl = wave + j * (kRT / 64);
      const int len = lens[j];
      const uint16_t* cp = cps[j];
      const double* vp = vps[j];
      double acc[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) acc[t] = 0.0;
      auto round = [&](int c, double a) __attribute__((always_inline)) {
        const double2* zp = cur2 + c * RW;
        const double2 z0 = zp[pc0], z1 = zp[pc1], z2 = zp[pc2], z3 = zp[pc3];
        acc[0] += a * z0.x;
        acc[1] += a * z0.y;
        acc[2] += a * z1.x;
        acc[3] += a * z1.y;
        acc[4] += a * z2.x;
        acc[5] += a * z2.y;
        acc[6] += a * z3.x;
        acc[7] += a * z3.y;
      };
      auto mul_group = [&](const int (&c)[kSliceGroup], const double (&a)[kSliceGroup]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSliceGroup; ++u) round(c[u], a[u]);
      };
      auto mul_part = [&](const int (&c)[kSliceGroup], const double (&a)[kSliceGroup], int cnt)
                          __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kSliceGroup; ++u)
          if (u < cnt) round(c[u], a[u]);  // uniform over the wave
      };
      // the slice the wave turns to after this one
      const int jn = (j + 1 < kSliceOwn && j + 1 < nown) ? j + 1 : 0;
      int k = 0;
      while (k + 2 * kSliceGroup <= len) {
        load_group(cb, ab, cp, vp, k + kSliceGroup);
        mul_group(ca, aa);
        load_group(ca, aa, cp, vp, k + 2 * kSliceGroup);
        mul_group(cb, ab);
        k += 2 * kSliceGroup;
      }
      if (len - k >= kSliceGroup) {
        load_group(cb, ab, cp, vp, k + kSliceGroup);
        mul_group(ca, aa);
        load_group(ca, aa, cps[jn], vps[jn], 0);
        mul_part(cb, ab, len - k - kSliceGroup);
      } else {
        int ct[kSliceGroup];
        double at[kSliceGroup];
#pragma unroll
        for (int u = 0; u < kSliceGroup; ++u) {
          ct[u] = ca[u];
          at[u] = aa[u];
        }
        load_group(ca, aa, cps[jn], vps[jn], 0);
        mul_part(ct, at, len - k);
      }
      const int r = sl * kSliceRows + lane;
      if (r < nr) {  // the recurrence with the row's sum, stored over u- (only this lane reads or writes that row of it)
        const double2* own = cur2 + r * RW;
        double2* out = prev2 + r * RW;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int at = pcs[t];
          const double2 o = own[at], pv = out[at];
          double2 w;
          w.x = alpha * (acc[2 * t] - shift * o.x) - beta * pv.x;
          w.y = alpha * (acc[2 * t + 1] - shift * o.y) - beta * pv.y;
          out[at] = w;
        }
      }
    }
    __syncthreads();  // every row of the new iterate is in place; nobody reads the old u- any more
    double* t = cur;
    cur = prev;
    prev = t;
  }
  for (int idx = tid; idx < nr * BS; idx += kRT) {
    const int r = idx / BS, t = idx - r * BS;
    y[(int64_t)(row0 + r) * ldy + col0 + t] = cur[idx];
  }
}

__global__ __launch_bounds__(kRT) void cheb_resident_kernel(const int64_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ col,
                                                            const double* __restrict__ val,
                                                            const double* __restrict__ x, double* __restrict__ y,
                                                            int64_t ldy, int b, int d, double alpha_first,
                                                            double alpha_rest, double shift,
                                                            const int32_t* __restrict__ items,
                                                            const uint16_t* __restrict__ scol,
                                                            const double* __restrict__ sval,
                                                            const int64_t* __restrict__ slice_base,
                                                            const int32_t* __restrict__ slice_len, int d32,
                                                            uint64_t rnd_key, int use_rnd) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int32_t* it = items + 4 * (int64_t)blockIdx.x;
  const int row0 = it[0], nr = it[1], col0 = it[2], cl = it[3] & 15, nx = it[3] >> 4;  // uniform over the workgroup
  if (cl == 4)
    resident_item<4>(rowptr, col, val, x, y, ldy, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, nx, smem, d32, rnd_key, use_rnd);
  else if (cl == 2)
    resident_item<2>(rowptr, col, val, x, y, ldy, b, d, alpha_first, alpha_rest, shift, row0, nr, col0, nx, smem, d32, rnd_key, use_rnd);
  else if (cl == 1)  // sliced form: the item's last word carries its first slice instead of a chunk count
    resident_item_sliced(scol, sval, slice_base, slice_len, x, y, ldy, b, d, alpha_first, alpha_rest, shift, row0, nr, col0,
                         nx, smem, rnd_key, use_rnd);
}

// ---- sliced copy of diagonal blocks ------------------------------------------------------------------------------------
// One wave per slice (64 consecutive rows of one block, fewer at the block's end).  slice_len = the longest row;
// slice_entries = 64 * slice_len: what the slice takes in the copy.
__global__ __launch_bounds__(256) void slice_len_kernel(const int64_t* __restrict__ rowptr,
                                                        const int32_t* __restrict__ slice_row0,
                                                        const int32_t* __restrict__ slice_rows, int nslices,
                                                        int32_t* __restrict__ slice_len,
                                                        int64_t* __restrict__ slice_entries) {
  const int sidx = (int)(((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (sidx >= nslices) return;
  const int64_t r = (int64_t)slice_row0[sidx] + lane;
  int len = lane < slice_rows[sidx] ? (int)(rowptr[r + 1] - rowptr[r]) : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const int other = __shfl_xor(len, o, 64);
    len = len > other ? len : other;
  }
  if (lane == 0) {
    slice_len[sidx] = len;
    slice_entries[sidx] = (int64_t)kSliceRows * len;
  }
}

// Fills slice sidx of the copy: round k of lane l sits at slice_base + 64 k + l.  Columns are stored relative to the
// block's first row (slice_blk0); the padding (rounds past a row's end, lanes past the block's end) has value 0.
//
// The order of a row's entries is chosen for the LDS banks.  In a round the 16 lanes of a pass read 16 bytes each from
// an operand row of 64 bytes: piece (t + lane) mod 4 of row c sits at bank quad 4 (c mod 4) + piece, so the four lanes
// of a pass that share a piece number must read rows that differ mod 4, or the pass is served in several turns.
// Lane l therefore puts into round k, while it has one, an entry whose column is ((l >> 2) + k) mod 4 modulo 4 (four
// cursors walk the row, one per residue class, each in the row's own order), else an entry of the next class that has
// any left; padding entries name a row of the wanted class.  The order depends on the matrix alone, so the sums stay
// reproducible.
__global__ __launch_bounds__(256) void slice_fill_kernel(const int64_t* __restrict__ rowptr,
                                                         const int32_t* __restrict__ col,
                                                         const double* __restrict__ val,
                                                         const int32_t* __restrict__ slice_row0,
                                                         const int32_t* __restrict__ slice_rows,
                                                         const int32_t* __restrict__ slice_blk0,
                                                         const int32_t* __restrict__ slice_blk_rows, int nslices,
                                                         const int64_t* __restrict__ slice_base,
                                                         const int64_t* __restrict__ slice_entries,
                                                         uint16_t* __restrict__ scol, double* __restrict__ sval) {
  const int sidx = (int)(((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (sidx >= nslices) return;
  const int rounds = (int)(slice_entries[sidx] / kSliceRows);
  const int64_t base = slice_base[sidx];
  const bool live = lane < slice_rows[sidx];
  const int64_t r = (int64_t)slice_row0[sidx] + lane;
  const int64_t e0 = live ? rowptr[r] : 0, e1 = live ? rowptr[r + 1] : 0;
  const int blk0 = slice_blk0[sidx];
  const unsigned last = (unsigned)(slice_blk_rows[sidx] - 1);
  auto local = [&](int64_t e) -> unsigned {
    const unsigned lc = (unsigned)(col[e] - blk0);
    return lc < last ? lc : last;  // a column outside the block (there is none in a diagonal block) stays inside LDS
  };
  auto next_of_class = [&](int64_t from, unsigned cls) -> int64_t {
    int64_t e = from;
    while (e < e1 && (local(e) & 3u) != cls) ++e;
    return e;
  };
  int64_t cur[4];
#pragma unroll
  for (unsigned cls = 0; cls < 4; ++cls) cur[cls] = next_of_class(e0, cls);
  for (int k = 0; k < rounds; ++k) {
    const unsigned want = (unsigned)((lane >> 2) + k) & 3u;
    unsigned lc = want <= last ? want : 0;  // padding: a row of the wanted class
    double av = 0.0;
#pragma unroll
    for (unsigned o = 0; o < 4; ++o) {
      const unsigned cls = (want + o) & 3u;
      bool took = false;
#pragma unroll
      for (unsigned q = 0; q < 4; ++q)  // cur[] is indexed with constants only (it lives in registers)
        if (q == cls && cur[q] < e1 && !took) {
          lc = local(cur[q]);
          av = val[cur[q]];
          cur[q] = next_of_class(cur[q] + 1, q);
          took = true;
        }
      if (took) break;
    }
    scol[base + (int64_t)k * kSliceRows + lane] = (uint16_t)lc;
    sval[base + (int64_t)k * kSliceRows + lane] = av;
  }
}

// extra[2 t] / extra[2 t + 1] = chunks beyond the first, summed over the rows of diagonal block t, for chunks of 32 /
// of 16 entries.  One wave per block.
__global__ __launch_bounds__(256) void block_extra_chunks_kernel(const int64_t* __restrict__ rowptr,
                                                                 const int32_t* __restrict__ starts, int nblk, int64_t n,
                                                                 int32_t* __restrict__ extra) {
  const int t = (int)(((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6);
  const int lane = threadIdx.x & 63;
  if (t >= nblk) return;
  const int64_t r0 = starts[t], r1 = t + 1 < nblk ? (int64_t)starts[t + 1] : n;
  int x32 = 0, x16 = 0;
  for (int64_t r = r0 + lane; r < r1; r += 64) {
    const int len = (int)(rowptr[r + 1] - rowptr[r]);
    if (len > 32) x32 += (len + 31) / 32 - 1;
    if (len > 16) x16 += (len + 15) / 16 - 1;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    x32 += __shfl_xor(x32, o, 64);
    x16 += __shfl_xor(x16, o, 64);
  }
  if (lane == 0) {
    extra[2 * t] = x32;
    extra[2 * t + 1] = x16;
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

size_t resident_item_lds_bytes(int nrows, int cl, int extra) { return resident_lds_bytes(nrows, cl, extra); }

int resident_max_chunks(int cl) { return kRS * (kRT / cl); }

int resident_slice_rows() { return kSliceRows; }

int64_t sliced_copy_tail_entries() { return (int64_t)3 * kSliceGroup * kSliceRows; }

size_t resident_sliced_lds_bytes(int nrows) {
  if (nrows > kSliceOwn * (kRT / 64) * kSliceRows) return ~(size_t)0;  // more slices than the waves own: no item
  return ((size_t)2 * nrows * 8 * sizeof(double) + 15) / 16 * 16;
}

size_t sliced_scan_workspace(int nslices) {
  size_t t = 0;
  (void)rocprim::exclusive_scan(nullptr, t, (int64_t*)nullptr, (int64_t*)nullptr, (int64_t)0, (size_t)nslices + 1,
                                rocprim::plus<int64_t>());
  return up256(t) + 256;
}

hipError_t sliced_copy_layout(const int64_t* rowptr, const int32_t* slice_row0, const int32_t* slice_rows, int nslices,
                              int32_t* slice_len, int64_t* slice_entries, int64_t* slice_base, void* work,
                              size_t work_bytes, hipStream_t st) {
  if (nslices <= 0) return hipSuccess;
  hipLaunchKernelGGL(slice_len_kernel, dim3((unsigned)(((int64_t)nslices * 64 + 255) / 256)), dim3(256), 0, st, rowptr,
                     slice_row0, slice_rows, nslices, slice_len, slice_entries);
  // slice_entries has nslices + 1 slots, the last one zero: the scan's last output is the copy's size
  hipError_t e = hipMemsetAsync(slice_entries + nslices, 0, sizeof(int64_t), st);
  if (e != hipSuccess) return e;
  e = rocprim::exclusive_scan(work, work_bytes, slice_entries, slice_base, (int64_t)0, (size_t)nslices + 1,
                              rocprim::plus<int64_t>(), st);
  if (e != hipSuccess) return e;
  return hipGetLastError();
}

hipError_t sliced_copy_fill(const int64_t* rowptr, const int32_t* col, const double* val, const int32_t* slice_row0,
                            const int32_t* slice_rows, const int32_t* slice_blk0, const int32_t* slice_blk_rows,
                            int nslices, const int64_t* slice_base, const int64_t* slice_entries, uint16_t* scol,
                            double* sval, hipStream_t st) {
  if (nslices <= 0) return hipSuccess;
  hipLaunchKernelGGL(slice_fill_kernel, dim3((unsigned)(((int64_t)nslices * 64 + 255) / 256)), dim3(256), 0, st, rowptr,
                     col, val, slice_row0, slice_rows, slice_blk0, slice_blk_rows, nslices, slice_base, slice_entries,
                     scol, sval);
  return hipGetLastError();
}

hipError_t launch_block_extra_chunks(const int64_t* rowptr, const int32_t* starts, int nblk, int64_t n, int32_t* extra,
                                     hipStream_t st) {
  if (nblk <= 0) return hipSuccess;
  hipLaunchKernelGGL(block_extra_chunks_kernel, dim3((unsigned)(((int64_t)nblk * 64 + 255) / 256)), dim3(256), 0, st,
                     rowptr, starts, nblk, n, extra);
  return hipGetLastError();
}

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
                                int64_t ldy, int b, int d, double alpha_first, double alpha_rest, double shift, const int32_t* items,
                                int nitems, size_t lds_bytes, const uint16_t* scol, const double* sval,
                                const int64_t* slice_base, const int32_t* slice_len, hipStream_t st, int d32,
                                uint64_t rnd_key, int use_rnd) {
  if (nitems <= 0 || d <= 0) return hipSuccess;
  if (d32 < 0 || d32 >= d) return hipErrorInvalidValue;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&cheb_resident_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(cheb_resident_kernel, dim3((unsigned)nitems), dim3(kRT), lds_bytes, st, rowptr, col, val, x, y, ldy, b, d,
                     alpha_first, alpha_rest, shift, items, scol, sval, slice_base, slice_len, d32, rnd_key, use_rnd);
  return hipGetLastError();
}

}  // namespace sceig
