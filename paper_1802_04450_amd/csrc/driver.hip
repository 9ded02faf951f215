// Host driver and C ABI (see include/sceig.h).
//
// Block Lanczos with full reorthogonalization, thick restart, locking and random re-injection for the
// largest eigenvalues of S = D^-1/2 W D^-1/2 (Section IV-B / Algorithm 3 of the paper, moved onto the
// GPU).  Everything of size n runs in the kernels of kernels.hip; this file only sequences them and
// solves the small projected eigenproblems (sym_eig.cpp).
//
// Basis layout: one row-major buffer of n rows and ld >= m + b columns.  Columns [0, nl) hold locked
// Ritz vectors, [nl, nl + ja) the active block-Krylov basis of the current phase, [nl + ja, nl + ja + b)
// the block being built.  A block step never leaves the device:
//   W = S V_last (SpMM) -> CGS2 against columns [0, nl + ja) (two MFMA projections + two MFMA updates)
//   -> Cholesky QR twice (Gram by MFMA, b x b factorisation in one workgroup) -> next block + its
//   scaled packed copy for the next SpMM.
// Per step the b x b diagonal block, the QR factor R and the Gram matrix of the residual block are
// kept in device "slots" and fetched only when the host inspects convergence.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <map>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "../../include/sceig.h"
#include "kernels.h"
#include "sym_eig.h"

namespace sceig {
namespace {

struct ScError {
  int code;
};

bool debug_on() {
  static const bool on = std::getenv("SCEIG_DEBUG") != nullptr;
  return on;
}

#define SC_THROW(code_)                                                                  \
  do {                                                                                   \
    if (debug_on()) std::fprintf(stderr, "[sceig] error %d at %s:%d\n", (code_), __FILE__, __LINE__); \
    throw ScError{(code_)};                                                              \
  } while (0)

#define HIP_TRY(expr)                                                                              \
  do {                                                                                             \
    hipError_t e__ = (expr);                                                                       \
    if (e__ != hipSuccess) {                                                                       \
      (void)hipGetLastError();                                                                     \
      if (debug_on())                                                                              \
        std::fprintf(stderr, "[sceig] %s failed: %s (%s:%d)\n", #expr, hipGetErrorString(e__), __FILE__, __LINE__); \
      throw ScError{e__ == hipErrorOutOfMemory ? SC_ENOMEM : SC_EHIP};                             \
    }                                                                                              \
  } while (0)

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// Device and pinned-host blocks released by a call are kept for the next call instead of going back to the driver
// (hipMalloc / hipFree / hipHostMalloc cost tens of microseconds each and hipFree synchronises the device; a solve
// makes about thirty of them).  A block is reused only for a request of exactly its size on the same device, which is
// what repeated solves of one problem shape ask for.  Every entry point synchronises its stream before it returns (and
// a call that fails waits for the device before its blocks are released, see settle_before_release), so no kernel of
// the releasing call can still be using a block when it is handed out again.  The cache holds at most
// `limit` bytes per kind (default 4 GiB, SCEIG_CACHE_LIMIT_MB overrides, 0 switches caching off); sc_release_cache()
// empties it.
class BlockCache {
 public:
  explicit BlockCache(bool pinned) : pinned_(pinned) {
    const char* e = std::getenv("SCEIG_CACHE_LIMIT_MB");
    limit_ = e ? (size_t)std::strtoull(e, nullptr, 10) << 20 : (size_t)4 << 30;
  }
  hipError_t get(size_t bytes, void** p) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    {
      std::lock_guard<std::mutex> lock(mu_);
      auto range = blocks_.equal_range(bytes);
      for (auto it = range.first; it != range.second; ++it) {
        if (it->second.dev == dev) {
          *p = it->second.p;
          blocks_.erase(it);
          held_ -= bytes;
          return hipSuccess;
        }
      }
    }
    return pinned_ ? hipHostMalloc(p, bytes, hipHostMallocDefault) : hipMalloc(p, bytes);
  }
  void put(void* p, size_t bytes) {
    int dev = 0;
    (void)hipGetDevice(&dev);
    {
      std::lock_guard<std::mutex> lock(mu_);
      if (held_ + bytes <= limit_) {
        blocks_.emplace(bytes, Block{p, dev});
        held_ += bytes;
        return;
      }
    }
    if (pinned_) {
      (void)hipHostFree(p);
    } else {
      (void)hipFree(p);
    }
  }
  void clear() {
    std::lock_guard<std::mutex> lock(mu_);
    int cur = 0;
    (void)hipGetDevice(&cur);
    for (auto& kv : blocks_) {
      if (pinned_) {
        (void)hipHostFree(kv.second.p);
      } else {
        (void)hipSetDevice(kv.second.dev);
        (void)hipFree(kv.second.p);
      }
    }
    (void)hipSetDevice(cur);
    blocks_.clear();
    held_ = 0;
  }

 private:
  struct Block {
    void* p;
    int dev;
  };
  bool pinned_;
  size_t limit_ = 0, held_ = 0;
  std::mutex mu_;
  std::multimap<size_t, Block> blocks_;
};

BlockCache& device_cache() {
  static BlockCache* c = new BlockCache(false);  // never destroyed: the HIP runtime may be gone at exit
  return *c;
}
BlockCache& pinned_cache() {
  static BlockCache* c = new BlockCache(true);
  return *c;
}

// A caller-provided workspace: while one is installed on the calling thread every device block of the call is carved
// out of it instead of coming from the cache, and nothing is allocated.  Blocks are 256-byte aligned and handed out
// bottom-up; a released block is reclaimed as soon as everything above it has been released too (the solver's blocks
// live in nested scopes, so the high-water mark stays at the sum of the blocks alive at one time).
class Arena {
 public:
  Arena(void* base, size_t bytes) {
    const uintptr_t b = reinterpret_cast<uintptr_t>(base), a = (b + 255) / 256 * 256;
    base_ = reinterpret_cast<char*>(a);
    cap_ = bytes > a - b ? bytes - (a - b) : 0;
  }
  void* get(size_t bytes) {
    const size_t need = (bytes + 255) / 256 * 256;
    if (need > cap_ - top_) return nullptr;
    void* p = base_ + top_;
    live_.push_back(Block{top_, need, false});
    top_ += need;
    peak_ = std::max(peak_, top_);
    return p;
  }
  void put(void* p) {
    const size_t off = (size_t)(static_cast<char*>(p) - base_);
    for (auto it = live_.rbegin(); it != live_.rend(); ++it)
      if (it->off == off) {
        it->freed = true;
        break;
      }
    while (!live_.empty() && live_.back().freed) {
      top_ = live_.back().off;
      live_.pop_back();
    }
  }
  size_t peak() const { return peak_; }

 private:
  struct Block {
    size_t off, bytes;
    bool freed;
  };
  char* base_ = nullptr;
  size_t cap_ = 0, top_ = 0, peak_ = 0;
  std::vector<Block> live_;
};
thread_local Arena* tl_arena = nullptr;

// Blocks that go back to the cache while an exception unwinds the call may still be in use by kernels the call had
// enqueued before it failed (the normal path synchronises its stream before it returns; the error path has not got
// there).  Waiting for the device first keeps a concurrent call on another stream from being handed such a block.
inline void settle_before_release() {
  if (std::uncaught_exceptions() > 0) (void)hipDeviceSynchronize();
}

template <typename T>
struct DevBuf {
  T* p = nullptr;
  size_t bytes = 0;
  Arena* arena = nullptr;
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
  void alloc(size_t count) {
    release();
    if (count == 0) count = 1;
    void* q = nullptr;
    if (tl_arena) {
      q = tl_arena->get(count * sizeof(T));
      if (!q) SC_THROW(SC_ENOMEM);  // the caller's workspace is too small
      arena = tl_arena;
    } else {
      HIP_TRY(device_cache().get(count * sizeof(T), &q));
    }
    p = static_cast<T*>(q);
    bytes = count * sizeof(T);
  }
  void release() {
    if (p) {
      if (arena) {
        arena->put(p);
      } else {
        settle_before_release();
        device_cache().put(p, bytes);
      }
    }
    p = nullptr;
    bytes = 0;
    arena = nullptr;
  }
  ~DevBuf() { release(); }
};

template <typename T>
struct PinnedBuf {
  T* p = nullptr;
  size_t bytes = 0;
  PinnedBuf() = default;
  PinnedBuf(const PinnedBuf&) = delete;
  PinnedBuf& operator=(const PinnedBuf&) = delete;
  void alloc(size_t count) {
    release();
    if (count == 0) count = 1;
    void* q = nullptr;
    HIP_TRY(pinned_cache().get(count * sizeof(T), &q));
    p = static_cast<T*>(q);
    bytes = count * sizeof(T);
  }
  void release() {
    if (p) {
      settle_before_release();
      pinned_cache().put(p, bytes);
    }
    p = nullptr;
    bytes = 0;
  }
  ~PinnedBuf() { release(); }
};

// Optional per-launch timing of selected kernel families with HIP events on the solver's stream.
enum Family { kFamSpmm = 0, kFamProject = 1, kFamUpdate = 2, kFamRotate = 3, kFamQr = 4, kFamOther = 5 };
struct KTimer {
  uint32_t mask = 0;
  hipStream_t st = nullptr;
  struct Rec {
    int fam;
    hipEvent_t a, b;
    double bytes, flops;
    int launches;
  };
  std::vector<Rec> recs;
  hipEvent_t cur = nullptr;
  bool on(int fam) const { return (mask >> fam) & 1u; }
  void begin(int fam) {
    if (!on(fam)) return;
    HIP_TRY(hipEventCreate(&cur));
    HIP_TRY(hipEventRecord(cur, st));
  }
  // bytes, flops: totals of the `launches` back-to-back launches between begin() and this call
  void end(int fam, double bytes, double flops, int launches = 1) {
    if (!on(fam)) return;
    hipEvent_t e;
    HIP_TRY(hipEventCreate(&e));
    HIP_TRY(hipEventRecord(e, st));
    recs.push_back(Rec{fam, cur, e, bytes, flops, launches});
    cur = nullptr;
  }
  // after the stream has been synchronised
  void collect(sc_stats* out) {
    for (Rec& r : recs) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
        out->fam_time_s[r.fam] += (double)ms * 1e-3;
        out->fam_launches[r.fam] += r.launches;
        out->fam_bytes[r.fam] += r.bytes;
        out->fam_flops[r.fam] += r.flops;
      }
      (void)hipEventDestroy(r.a);
      (void)hipEventDestroy(r.b);
    }
    recs.clear();
  }
  ~KTimer() {
    for (Rec& r : recs) {
      (void)hipEventDestroy(r.a);
      (void)hipEventDestroy(r.b);
    }
    if (cur) (void)hipEventDestroy(cur);
  }
};

constexpr int kPP = kPartialPad;
constexpr int kSlotDoubles = 3 * kPP * kPP;  // A, R, G
constexpr int kMaxPartials = 512;
constexpr double kAbsDrop2 = 1e-24;  // squared norm below which a residual column counts as zero
constexpr double kRelDrop = 1e-12;   // squared sine below which a column counts as dependent

int pow2_floor(int x) {
  int p = 1;
  while (p * 2 <= x) p *= 2;
  return p;
}

// CGS2 of basis[:, wcol : wcol+b] against basis[:, 0 : j]; hsum (j x b, stride kPP) = H1 + H2.
// The second pass runs against columns [second_from, j) only (0 = all of them, the plain CGS2).  The solver
// passes the number of locked vectors here: the block's components along locked eigenvectors are of the order of
// their residuals, so removing them once involves no cancellation, whereas the active Krylov vectors, which take
// most of the block's norm away, get the second pass.
// slot_a (may be null) receives rows [slot_row0, j) of hsum after the last pass.  If gpart != null the last update also leaves
// the Gram partials of the updated block there; returns their count (0 if none were produced).
// first_from > 0: the first pass too leaves the columns before it alone (the solver's tentative first step).
// gram_only: the last update (against fewer than kWideUpdate columns) is made for the Gram partials alone and the block
// itself is not stored back (a block that will be dropped or built again).
constexpr int kWideUpdate = 256;  // contraction lengths from which update + separate Gram beats the fused kernel

int enqueue_cgs2(double* basis, int64_t n, int64_t ld, int j, int wcol, int b, int second_from, double* part,
                 double* h1, double* hsum, double* slot_a, int slot_row0, double* gpart, hipStream_t st, KTimer* tm,
                 int first_from = 0, bool gram_only = false) {
  if (j <= 0) return 0;
  KTimer none;
  if (!tm) tm = &none;
  // algorithmic traffic of one pass over the basis: every row reads its basis entries and its b block
  // entries once (the update also writes the b block entries back)
  const double rows = (double)n;
  int ngram = 0;
  for (int pass = 0; pass < 2; ++pass) {
    const int c0 = pass == 0 ? first_from : second_from;  // first basis column of this pass
    const int jc = j - c0;
    if (jc <= 0) {  // nothing to do in this pass: the Gram partials then come from the block QR itself
      continue;
    }
    const ProjectPlan plan = plan_project(n, jc, kMaxPartials);
    tm->begin(kFamProject);
    HIP_TRY(launch_project(basis, n, ld, c0, jc, wcol, b, plan, part, st));
    tm->end(kFamProject, 8.0 * rows * (jc + b), 2.0 * rows * jc * b);
    const bool last_pass = pass == 1 || j - second_from <= 0;  // the last update leaves the Gram partials
    tm->begin(kFamOther);
    HIP_TRY(launch_reduce_partials(part, plan.npart, jc, b, h1, hsum + (size_t)c0 * kPP, pass,
                                   last_pass ? slot_a : nullptr, slot_row0 - c0, st));
    tm->end(kFamOther, 8.0 * plan.npart * (double)jc * b, 0.0);
    tm->begin(kFamUpdate);
    if (last_pass && gpart && jc >= kWideUpdate) {
      // against many columns the plain update is the faster kernel (more waves in flight: at n = 500,000 and 1,024
      // columns 995 against 1,300 us), and the Gram partials of the updated block cost one pass over the block alone
      HIP_TRY(launch_row_gemm(basis, n, ld, c0, jc, h1, kPP, b, 0, wcol, nullptr, 0, nullptr, st));
      const ProjectPlan gplan = plan_project(n, b, kMaxPartials);
      HIP_TRY(launch_project(basis, n, ld, wcol, b, wcol, b, gplan, gpart, st));
      ngram = gplan.npart;
    } else if (last_pass && gpart) {
      HIP_TRY(launch_update_gram(basis, n, ld, c0, jc, h1, b, wcol, gram_only ? 2 : 0, gpart, st));
      ngram = plan_update_gram(n);
    } else {
      HIP_TRY(launch_row_gemm(basis, n, ld, c0, jc, h1, kPP, b, 0, wcol, nullptr, 0, nullptr, st));
    }
    tm->end(kFamUpdate, 8.0 * rows * (jc + 2 * b), 2.0 * rows * jc * b);
  }
  return ngram;
}

// Gram-Schmidt of basis[:, wcol : wcol+b] against basis[:, 0 : j] with the second pass decided on the device ("twice
// is enough", and once is when nothing is lost to cancellation): after the first pass a one-workgroup kernel compares,
// per column, the squared norm the pass removed with the squared norm it kept; if no column lost more than a factor
// 10^6 (orthogonality error after one pass about 1e-16 * 1e3), the three launches of the second pass find skip[0] set
// and return at once.  No host round trip either way.  gpart receives the Gram partials of the final block (from the
// first update, overwritten by the second when it runs); returns their count.  gram_tmp: kPP*kPP doubles of scratch.
int enqueue_cgs_adaptive(double* basis, int64_t n, int64_t ld, int j, int wcol, int b, double* part, double* h1,
                         double* hsum, double* gpart, double* gram_tmp, int* skip, hipStream_t st, KTimer* tm) {
  if (j <= 0) return 0;
  KTimer none;
  if (!tm) tm = &none;
  const double rows = (double)n;
  const ProjectPlan plan = plan_project(n, j, kMaxPartials);
  const ProjectPlan gplan = plan_project(n, b, kMaxPartials);
  const bool wide = j >= kWideUpdate;
  const int ngram = wide ? gplan.npart : plan_update_gram(n);
  for (int pass = 0; pass < 2; ++pass) {
    const int* sk = pass == 0 ? nullptr : skip;
    // the second pass's traffic is not counted: whether it ran is known on the device only
    const double counted = pass == 0 ? 1.0 : 0.0;
    tm->begin(kFamProject);
    HIP_TRY(launch_project(basis, n, ld, 0, j, wcol, b, plan, part, st, sk));
    tm->end(kFamProject, counted * 8.0 * rows * (j + b), counted * 2.0 * rows * j * b);
    tm->begin(kFamOther);
    HIP_TRY(launch_reduce_partials(part, plan.npart, j, b, h1, hsum, pass, nullptr, 0, st, sk));
    tm->end(kFamOther, counted * 8.0 * plan.npart * (double)j * b, 0.0);
    tm->begin(kFamUpdate);
    if (wide) {  // see enqueue_cgs2
      HIP_TRY(launch_row_gemm(basis, n, ld, 0, j, h1, kPP, b, 0, wcol, nullptr, 0, nullptr, st, sk));
      HIP_TRY(launch_project(basis, n, ld, wcol, b, wcol, b, gplan, gpart, st, sk));
    } else {
      HIP_TRY(launch_update_gram(basis, n, ld, 0, j, h1, b, wcol, 0, gpart, st, sk));
    }
    tm->end(kFamUpdate, counted * 8.0 * rows * (j + 2 * b), counted * 2.0 * rows * j * b);
    if (pass == 0) {
      HIP_TRY(launch_reduce_partials(gpart, ngram, b, b, gram_tmp, nullptr, 0, nullptr, 0, st));
      HIP_TRY(launch_second_pass_test(h1, j, b, gram_tmp, 1e6, skip, st));
    }
  }
  return ngram;
}

// Cholesky QR twice on basis[:, col : col+b].  r_out / g_out: device b x b (stride kPP) or null;
// gram, rinv, r1: device scratch of kPP*kPP doubles each; gpart: scratch for Gram partials (kGramPartials blocks).
// ngram > 0: gpart already holds that many Gram partials of the block (left by enqueue_cgs2).
// z (may be null): packed s-scaled copy of the orthonormalised block.
void enqueue_block_qr(double* basis, int64_t n, int64_t ld, int col, int b, double* part, double* gpart, int ngram,
                      double* gram, double* rinv, double* r1, double* r_out, double* g_out, double* z, const double* s,
                      hipStream_t st, KTimer* tm) {
  KTimer none;
  if (!tm) tm = &none;
  const double blk = 8.0 * (double)n * b;
  tm->begin(kFamQr);
  if (ngram > 0) {
    HIP_TRY(launch_reduce_partials(gpart, ngram, b, b, gram, nullptr, 0, nullptr, 0, st));
  } else {
    const ProjectPlan plan = plan_project(n, b, kMaxPartials);
    HIP_TRY(launch_project(basis, n, ld, col, b, col, b, plan, part, st));
    HIP_TRY(launch_reduce_partials(part, plan.npart, b, b, gram, nullptr, 0, nullptr, 0, st));
  }
  HIP_TRY(launch_gram_cholesky(gram, b, g_out, rinv, r1, nullptr, kAbsDrop2, kRelDrop, st));
  HIP_TRY(launch_update_gram(basis, n, ld, col, b, rinv, b, col, 1, gpart, st));
  HIP_TRY(launch_reduce_partials(gpart, plan_update_gram(n), b, b, gram, nullptr, 0, nullptr, 0, st));
  // second pass: a column that survived the first pass has unit norm, so only exact zeros are dropped
  HIP_TRY(launch_gram_cholesky(gram, b, nullptr, rinv, r_out, r1, 0.25, 1e-8, st));
  HIP_TRY(launch_apply_rinv(basis, n, ld, col, b, rinv, z, s, st));
  tm->end(kFamQr, (ngram > 0 ? 4.0 : 5.0) * blk + (z ? blk : 0.0), 4.0 * (double)n * b * b);
}

std::atomic<int64_t> resident_launches{0};  // sc_counter(SC_COUNTER_RESIDENT_FILTERS)

// Plan of the LDS-resident Chebyshev filter (resident.hip) for one matrix and block width: the diagonal blocks of the
// matrix cut into work items (block rows x column slice) whose two iterates fit the LDS of a compute unit.
struct ResidentPlan {
  DevBuf<int32_t> items;
  int nitems = 0;
  size_t lds_bytes = 0;
  bool usable = false;
  double est_step_s = 0.0;  // modelled time of one recurrence step
  int64_t rest_row0 = 0;    // rows [rest_row0, n): blocks that fit no item, left to the product-per-step kernel
  // sliced copy of the blocks that are worked on in the sliced form (null if there are none)
  DevBuf<uint16_t> scol;
  DevBuf<double> sval;
  DevBuf<int64_t> slice_base;
  DevBuf<int32_t> slice_len;
};

int device_lds_limit() {
  int dev = 0, lds = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
  return lds;
}

// Finds the diagonal blocks and their chunk counts on the device, sizes the items on the host.  A block goes, in this
// order of preference, as items of 32 or 16 columns with its entries in registers (at most two chunks per lane
// group), or as 8-column items in the sliced form (entries streamed from a sliced copy made here from `val`).  The
// plan is usable when b is 16 or 32, every block fits LDS one way or the other, the sliced copy's padding stays below
// a half, and the modelled step time beats the general product's: an item costs the LDS bytes its step reads (entries
// times 8 bytes per column; the sliced form's streamed entries are charged as 48 more bytes each) at about half a
// compute unit's LDS rate, the items spread over the 256 compute units, largest first; the general product gathers
// 8 b bytes per entry from the L2 caches at the 12.5 TB/s measured for it, and no launch is shorter than about 4 us.
void plan_resident(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, int64_t nnz, int b,
                   hipStream_t st, ResidentPlan* plan) {
  plan->usable = false;
  plan->nitems = 0;
  if ((b != 16 && b != 32) || n <= 0 || nnz <= 0 || std::getenv("SCEIG_NO_RESIDENT")) return;
  const int lds_limit = device_lds_limit() - 1024;
  if (lds_limit < 32 * 1024) return;
  const bool no_sliced = std::getenv("SCEIG_NO_SLICED") != nullptr;
  DevBuf<char> work;
  DevBuf<int32_t> starts, count, extra;
  const size_t wb = diagonal_blocks_workspace(n);
  work.alloc(wb);
  starts.alloc((size_t)n);
  count.alloc(1);
  HIP_TRY(diagonal_blocks(rowptr, col, n, work.p, wb, starts.p, count.p, st));
  int32_t nblk = 0;
  HIP_TRY(hipMemcpyAsync(&nblk, count.p, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (nblk <= 0 || (int64_t)nblk > (int64_t)1 << 22) return;  // the item table stays small
  extra.alloc((size_t)2 * nblk);
  HIP_TRY(launch_block_extra_chunks(rowptr, starts.p, nblk, n, extra.p, st));
  std::vector<int32_t> hs((size_t)nblk + 1), hx((size_t)2 * nblk);
  HIP_TRY(hipMemcpyAsync(hs.data(), starts.p, (size_t)nblk * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipMemcpyAsync(hx.data(), extra.p, (size_t)2 * nblk * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  hs[nblk] = (int32_t)n;
  struct Item {
    int32_t row0, nrows, col0, shape;
  };
  std::vector<Item> items;
  std::vector<int32_t> srow0, srows, sblk0, sblkrows;  // the slices of the blocks that go in the sliced form
  std::vector<int> sliced_blocks;
  const int srows_max = resident_slice_rows();
  size_t lds_max = 0;
  const double avg_deg = (double)nnz / (double)n;
  double sum_cost = 0.0, max_cost = 0.0;
  int64_t rest_row0 = n;
  for (int t = 0; t < nblk; ++t) {
    const int nr = hs[t + 1] - hs[t];
    int cl = 0, nx = 0;
    for (int c = b == 32 ? 4 : 2; c >= 2; c /= 2) {  // widest lane group first
      const int x = c == 4 ? hx[2 * t] : hx[2 * t + 1];
      if (x >= (1 << 26) || nr + x > resident_max_chunks(c)) continue;
      if (resident_item_lds_bytes(nr, c, x) > (size_t)lds_limit) continue;
      cl = c;
      nx = x;
      break;
    }
    if (cl == 0 && (no_sliced || nr > 65535 || resident_sliced_lds_bytes(nr) > (size_t)lds_limit)) {
      // fits no item: acceptable only as part of a run of such blocks at the end of the matrix (the solver's
      // renumbering puts the large components there), which the product-per-step kernel then takes
      if (rest_row0 == n) rest_row0 = hs[t];
      continue;
    }
    if (rest_row0 < n) return;  // an item after a block without one: the blocks without items are not a suffix
    if (cl == 0) {
      // the sliced form: column indices inside the block take 16 bits, the item's first slice 27
      if (srow0.size() + (size_t)nr / srows_max + 1 >= ((size_t)1 << 27)) return;
      cl = 1;
      nx = (int)srow0.size();
      for (int r = 0; r < nr; r += srows_max) {
        srow0.push_back(hs[t] + r);
        srows.push_back(std::min(srows_max, nr - r));
        sblk0.push_back(hs[t]);
        sblkrows.push_back(nr);
      }
      sliced_blocks.push_back(t);
    }
    const int bs = 8 * cl;
    const double cost = (double)nr * avg_deg * (8.0 * bs + (cl == 1 ? 48.0 : 0.0));
    for (int c0 = 0; c0 < b; c0 += bs) {
      items.push_back(Item{hs[t], nr, c0, (int32_t)(cl | (nx << 4))});
      sum_cost += cost;
    }
    max_cost = std::max(max_cost, cost);
    lds_max = std::max(lds_max, cl == 1 ? resident_sliced_lds_bytes(nr) : resident_item_lds_bytes(nr, cl, nx));
  }
  const double cu_rate = 150e9;  // bytes per second out of one compute unit's LDS, about half of its peak
  if (items.empty()) return;
  const double general_step_s = std::max(4e-6, (double)nnz * 8.0 * b / 12.5e12);
  // the rows without items still take the general product, step by step, after the one launch of the items
  const double rest_share = (double)(n - rest_row0) / (double)n;
  plan->est_step_s = std::max(max_cost, sum_cost / 256.0) / cu_rate + 1e-6 +
                     (rest_share > 0.0 ? std::max(4e-6, rest_share * general_step_s) : 0.0);
  if (debug_on())
    std::fprintf(stderr, "[sceig] resident filter plan: %d blocks (%zu sliced), %zu items, LDS %zu, modelled step %.1f us "
                 "against %.1f us\n", nblk, sliced_blocks.size(), items.size(), lds_max, plan->est_step_s * 1e6,
                 general_step_s * 1e6);
  if (!(plan->est_step_s < general_step_s) && !std::getenv("SCEIG_FORCE_RESIDENT")) return;
  const int nslices = (int)srow0.size();
  if (nslices > 0) {
    DevBuf<int32_t> d_row0, d_rows, d_blk0, d_blkrows;
    DevBuf<int64_t> d_entries;
    DevBuf<char> swork;
    d_row0.alloc((size_t)nslices);
    d_rows.alloc((size_t)nslices);
    d_blk0.alloc((size_t)nslices);
    d_blkrows.alloc((size_t)nslices);
    d_entries.alloc((size_t)nslices + 1);
    plan->slice_base.alloc((size_t)nslices + 1);
    plan->slice_len.alloc((size_t)nslices);
    const size_t sw = sliced_scan_workspace(nslices);
    swork.alloc(sw);
    const size_t ib = (size_t)nslices * sizeof(int32_t);
    HIP_TRY(hipMemcpyAsync(d_row0.p, srow0.data(), ib, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(d_rows.p, srows.data(), ib, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(d_blk0.p, sblk0.data(), ib, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(d_blkrows.p, sblkrows.data(), ib, hipMemcpyHostToDevice, st));
    HIP_TRY(sliced_copy_layout(rowptr, d_row0.p, d_rows.p, nslices, plan->slice_len.p, d_entries.p, plan->slice_base.p,
                               swork.p, sw, st));
    int64_t total = 0;
    HIP_TRY(hipMemcpyAsync(&total, plan->slice_base.p + nslices, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));  // also: the host vectors above have been read
    // padding: against the sliced blocks' share of the matrix entries, estimated by their share of the rows
    int64_t sliced_rows = 0;
    for (int t : sliced_blocks) sliced_rows += hs[t + 1] - hs[t];
    const double basis_entries = (double)nnz * (double)sliced_rows / (double)n;
    if (debug_on())
      std::fprintf(stderr, "[sceig] sliced copy: %d slices, %lld entries for %.0f of the matrix\n", nslices,
                   (long long)total, basis_entries);
    if ((double)total > 1.5 * basis_entries && !std::getenv("SCEIG_FORCE_RESIDENT")) {
      plan->slice_base.release();
      plan->slice_len.release();
      return;
    }
    const size_t tail = (size_t)sliced_copy_tail_entries();
    plan->scol.alloc((size_t)total + tail);
    plan->sval.alloc((size_t)total + tail);
    HIP_TRY(hipMemsetAsync(plan->scol.p + total, 0, tail * sizeof(uint16_t), st));
    HIP_TRY(hipMemsetAsync(plan->sval.p + total, 0, tail * sizeof(double), st));
    HIP_TRY(sliced_copy_fill(rowptr, col, val, d_row0.p, d_rows.p, d_blk0.p, d_blkrows.p, nslices, plan->slice_base.p,
                             d_entries.p, plan->scol.p, plan->sval.p, st));
    HIP_TRY(hipStreamSynchronize(st));  // the temporaries above are released on return
  }
  std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& c) {
    return (int64_t)a.nrows * (a.shape & 15) > (int64_t)c.nrows * (c.shape & 15);
  });
  {
    // Workgroups go to the eight XCDs in turn (workgroup i to XCD i mod 8), each XCD with an L2 of its own.  The items
    // of one block (its column slices) read the same matrix entries, so they are placed eight apart: they run on the
    // same XCD at about the same time, and what the first fetches the others find in that L2.
    std::vector<std::vector<Item>> queue(8);
    size_t q = 0;
    for (size_t i = 0; i < items.size();) {
      size_t j = i;
      while (j < items.size() && items[j].row0 == items[i].row0) ++j;
      for (size_t t = i; t < j; ++t) queue[q % 8].push_back(items[t]);
      ++q;
      i = j;
    }
    std::vector<Item> placed;
    placed.reserve(items.size());
    for (size_t r = 0; placed.size() < items.size(); ++r)
      for (int x = 0; x < 8; ++x)
        if (r < queue[x].size()) placed.push_back(queue[x][r]);
    items.swap(placed);
  }
  plan->items.alloc(items.size() * 4);
  HIP_TRY(hipMemcpyAsync(plan->items.p, items.data(), items.size() * sizeof(Item), hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));  // `items` is pageable host memory
  plan->nitems = (int)items.size();
  plan->lds_bytes = lds_max;
  plan->rest_row0 = rest_row0;
  plan->usable = true;
}

// Chebyshev filter of a packed block: result = T_d(g(S)) X, g the affine map taking [-1, a] to [-1, 1], by the
// three-term recurrence Y_0 = X, Y_1 = g(S) X, Y_{i+1} = 2 g(S) Y_i - Y_{i-1}; one sparse product per step.
//   wide blocks (val_scaled != null, b >= 8): z holds X packed; the recurrence is fused into the product kernel and
//     rotates through z, buf1 and buf2.
//   narrow blocks: z holds s o X packed and buf1 holds X packed; buf2 and buf3 are scratch (product + combine kernel).
// All buffers are packed n x b.  Returns the buffer that holds the result - or null when the one-launch form has
// written it to `direct` (n x b with leading dimension direct_ld; optional), which saves the caller a copy.
double* enqueue_cheb_filter(const int64_t* rowptr, const int32_t* col, const double* val, const double* val_scaled,
                            const double* s, int64_t n, int64_t nnz, int b, int d, double a, double* z, double* buf1,
                            double* buf2, double* buf3, double avg_deg, const int32_t* longrows, int nlong,
                            const ResidentPlan* resident, hipStream_t st, KTimer* tm, double* direct = nullptr,
                            int64_t direct_ld = 0, double lo = -1.0, int d32 = 0, uint64_t rnd_key = 0, int use_rnd = 0) {
  // lo: lower end of the damped interval; -1 always holds (||S||_2 = 1), the solver passes its estimate of the
  // bottom of the spectrum when it has one
  KTimer none;
  if (!tm) tm = &none;
  const double c = 0.5 * (a + lo), e = 0.5 * (a - lo);
  const double bytes = 12.0 * (double)nnz + 8.0 * (double)(n + 1) + (val_scaled ? 0.0 : 8.0 * (double)n) +
                       16.0 * (double)n * b;
  if (val_scaled && resident && resident->usable) {
    // all d steps in one launch, iterates in LDS: the matrix entries are streamed once per step and column slice, the
    // block is read once and written once
    resident_launches.fetch_add(1, std::memory_order_relaxed);
    double* out = direct ? direct : buf1;
    const int64_t ldo = direct ? direct_ld : (int64_t)b;
    tm->begin(kFamSpmm);
    HIP_TRY(launch_cheb_resident(rowptr, col, val_scaled, z, out, ldo, b, d, 1.0 / e, 2.0 / e, c, resident->items.p,
                                 resident->nitems, resident->lds_bytes, resident->scol.p, resident->sval.p,
                                 resident->slice_base.p, resident->slice_len.p, st, d32, rnd_key, use_rnd));
    const int64_t r0 = resident->rest_row0;
    if (r0 < n) {
      // the blocks without an item: the recurrence step by step on their rows alone (their iterates rotate through the
      // same three buffers, in rows the items do not touch), then into the result
      double* cur = z;
      double* prev = buf2;
      double* next = buf1;
      for (int i = 0; i < d; ++i) {
        HIP_TRY(launch_spmm_vals_cheb(rowptr, col, val_scaled, n, cur, b, prev, next, i == 0 ? 1.0 / e : 2.0 / e, c,
                                      i == 0 ? 0.0 : 1.0, avg_deg, longrows, nlong, st, r0));
        double* t = prev;
        prev = cur;
        cur = next;
        next = t;
      }
      if (cur != out)
        HIP_TRY(launch_copy_cols(cur + r0 * b, b, 0, out + r0 * ldo, ldo, 0, b, n - r0, st));
    }
    tm->end(kFamSpmm, d * bytes + (d - 1) * 8.0 * (double)n * b, d * 2.0 * (double)nnz * b, d);
    return direct ? nullptr : buf1;
  }
  if (val_scaled) {
    double* cur = z;
    double* prev = buf1;
    double* next = buf2;
    tm->begin(kFamSpmm);  // one event pair round the d back-to-back launches
    for (int i = 0; i < d; ++i) {
      HIP_TRY(launch_spmm_vals_cheb(rowptr, col, val_scaled, n, cur, b, prev, next, i == 0 ? 1.0 / e : 2.0 / e, c,
                                    i == 0 ? 0.0 : 1.0, avg_deg, longrows, nlong, st));
      double* t = prev;
      prev = cur;
      cur = next;
      next = t;
    }
    tm->end(kFamSpmm, d * bytes + (d - 1) * 8.0 * (double)n * b, d * 2.0 * (double)nnz * b, d);
    return cur;
  }
  double* ycur = buf1;
  double* yprev = buf2;
  for (int i = 0; i < d; ++i) {
    tm->begin(kFamSpmm);
    HIP_TRY(launch_spmm(rowptr, col, val, s, n, z, b, buf3, b, avg_deg, st));
    tm->end(kFamSpmm, bytes, 2.0 * (double)nnz * b);
    HIP_TRY(launch_cheb_combine(buf3, ycur, i == 0 ? ycur : yprev, s, i == 0 ? 1.0 / e : 2.0 / e, c, i == 0 ? 0.0 : 1.0,
                                yprev, z, n, b, st));
    std::swap(ycur, yprev);
  }
  return ycur;
}

constexpr int kGramPartials = 1024;

// Connected components by label propagation on the device, then rows and columns are renumbered so that every
// component is contiguous (stable inside a component).  The sparse products then gather from a few hundred KB at
// a time instead of from all over the vector; mathematically the result is a permutation similarity of the input.
// Outputs: permuted CSR (device, caller-allocated, same sizes as the input), old_of_new (device int32[n]: original
// index of each new row), optionally new_of_old (device int32[n], the inverse map) and the component index of each
// new row (host).  Returns the component count.
int reorder_csr(const int64_t* rowptr, const int32_t* col, const double* val, int64_t n, int64_t nnz,
                int64_t* rowptr_out, int32_t* col_out, double* val_out, int32_t* old_of_new_out,
                int32_t* new_of_old_out, std::vector<int32_t>* comp_of_new, int by_length, hipStream_t st,
                int big_rows = 0) {
  DevBuf<int32_t> label, new_of_old_own;
  DevBuf<int> flag;
  label.alloc((size_t)n);
  flag.alloc(1);
  HIP_TRY(launch_iota(label.p, n, st));
  for (int round = 0; round < 100000; ++round) {
    int h = 0;
    HIP_TRY(hipMemsetAsync(flag.p, 0, sizeof(int), st));
    HIP_TRY(launch_cc_round(rowptr, col, val, label.p, n, flag.p, st));
    HIP_TRY(launch_cc_round(rowptr, col, val, label.p, n, flag.p, st));
    HIP_TRY(hipMemcpyAsync(&h, flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (debug_on() && (round % 50 == 49)) std::fprintf(stderr, "[sceig] component pass: %d rounds\n", 2 * (round + 1));
    if (!h) break;
    if (round + 1 == 100000) SC_THROW(SC_EINTERNAL);  // labels still changing: they do not name the components yet
  }
  // numbering, permuted row pointers and component index of every new row, all on the device
  int32_t* new_of_old_dev = new_of_old_out;
  if (!new_of_old_dev) {
    new_of_old_own.alloc((size_t)n);
    new_of_old_dev = new_of_old_own.p;
  }
  DevBuf<char> work;
  DevBuf<int32_t> comp_dev;
  const size_t work_bytes = order_by_component_workspace(n);
  work.alloc(work_bytes);
  comp_dev.alloc((size_t)n);
  HIP_TRY(order_by_component(rowptr, col, label.p, n, by_length, big_rows, work.p, work_bytes, old_of_new_out, new_of_old_dev,
                             rowptr_out, comp_dev.p, st));
  HIP_TRY(launch_permute_csr(rowptr, col, val, old_of_new_out, new_of_old_dev, rowptr_out, col_out, val_out, n, st));
  int32_t last_comp = 0;
  HIP_TRY(hipMemcpyAsync(&last_comp, comp_dev.p + (n - 1), sizeof(int32_t), hipMemcpyDeviceToHost, st));
  if (comp_of_new) {
    comp_of_new->assign((size_t)n, 0);
    HIP_TRY(hipMemcpyAsync(comp_of_new->data(), comp_dev.p, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  }
  HIP_TRY(hipStreamSynchronize(st));
  const int ncomp = (int)last_comp + 1;
  (void)nnz;
  return ncomp;
}

// The projected matrix of a phase: m x m with a fixed leading dimension, zero pages from the system until touched.
// Only the leading square that has been written since the last clear() is cleared again (a phase rarely assembles more
// than a few blocks, while m x m can be 128 MB).
struct ProjectedMatrix {
  double* a = nullptr;
  size_t ld = 0;
  int hi = 0;  // rows and columns >= hi are zero
  ProjectedMatrix() = default;
  ProjectedMatrix(const ProjectedMatrix&) = delete;
  ProjectedMatrix& operator=(const ProjectedMatrix&) = delete;
  void init(int m) {
    a = static_cast<double*>(std::calloc((size_t)m * m, sizeof(double)));
    if (!a) throw std::bad_alloc();
    ld = (size_t)m;
  }
  double& at(int x, int y) { return a[(size_t)x * ld + y]; }
  void touch(int extent) { hi = std::max(hi, std::min(extent, (int)ld)); }
  void clear() {
    for (int x = 0; x < hi; ++x) std::memset(a + (size_t)x * ld, 0, sizeof(double) * hi);
    hi = 0;
  }
  ~ProjectedMatrix() { std::free(a); }
};

struct Solver {
  // problem
  const int64_t* rowptr;
  const int32_t* col;
  const double* val;
  int64_t n, nnz;
  int k;      // pairs the iteration works for: the caller's k plus the guard vectors
  int k_out;  // pairs returned
  double tol;
  int maxiter;
  // options
  int m, b, check_every;
  uint32_t flags;
  uint64_t seed;
  const double* v0 = nullptr;  // caller's start vector (caller's numbering), or null
  bool no_late_projection = std::getenv("SCEIG_NO_LATE_PROJECTION") != nullptr;
  bool no_spectrum_bottom = std::getenv("SCEIG_NO_SPECTRUM_BOTTOM") != nullptr;
  bool no_tentative_step = std::getenv("SCEIG_NO_TENTATIVE_STEP") != nullptr;
  bool no_resident_product = std::getenv("SCEIG_NO_RESIDENT_PRODUCT") != nullptr;
  bool no_random_inside = std::getenv("SCEIG_NO_RANDOM_INSIDE") != nullptr;
  // A start-block filter only prepares a block whose Ritz pairs the Lanczos step then tests in double precision.  In
  // its one-launch form all steps but the last filter_tail64 run in single precision (half the LDS traffic that bounds
  // the form): the later steps damp what the rounding of the earlier ones adds along the unwanted directions.
  // SCEIG_FILTER_FP64_TAIL = a number larger than any degree keeps every step in double precision.
  int filter_tail64 = std::getenv("SCEIG_FILTER_FP64_TAIL") ? std::atoi(std::getenv("SCEIG_FILTER_FP64_TAIL")) : 6;
  bool tentative_two_passes = std::getenv("SCEIG_TENTATIVE_TWO_PASSES") != nullptr;
  double tentative_min_work = std::getenv("SCEIG_TENTATIVE_MIN_WORK") ? std::atof(std::getenv("SCEIG_TENTATIVE_MIN_WORK")) : 2e7;
  size_t ws_limit = 0;         // > 0: size of the caller's workspace, checked against the estimate once nnz is known
  hipStream_t st;
  // device
  DevBuf<double> basis, s, z, part, gpart, h1, hsum, small, slots, yd, rot;
  DevBuf<int> flag;
  DevBuf<int64_t> rowptr_p;
  DevBuf<int32_t> col_p, old_of_new_d, new_of_old_d, comp_d, perm_d;
  DevBuf<double> val_p, coef_d;
  DevBuf<double> val_s;  // S_ij = s_i W_ij s_j multiplied out: the operator copy used when b >= 8
  DevBuf<int32_t> longrows;  // rows with more than kLongRow entries (wide products only), ascending
  int nlong = 0;
  ResidentPlan resident;     // LDS-resident start-block filter (wide products on a block-diagonal operator)
  const int32_t* rowmap = nullptr;  // device: original row of each internal row, null if not reordered
  const int32_t* rowinv = nullptr;  // device: internal row of each original row, null if not reordered
  std::vector<int32_t> comp_host;   // component index of each internal row (only after reorder())
  int ncomp = 0;
  PinnedBuf<double> slots_host;
  // pinned staging for the small coefficient blocks of a rotation (locking b Ritz vectors): the upload then needs no
  // wait on the host.  ystage_busy: an upload from it may still be in flight (cleared by the next wait on the stream).
  PinnedBuf<double> ystage;
  static constexpr size_t kYStageDoubles = 16384;
  bool ystage_busy = false;
  int64_t ld = 0;
  int max_slots = 0;
  size_t yd_cap = 0, rot_cols = 0;
  double avg_deg = 0;
  // state
  int nl = 0;
  std::vector<double> theta_locked, rho_locked;
  // Chebyshev filter of the next phase's start block: degree (0 = none) and upper end of the damped interval
  int filt_d = 0;
  double filt_a = 0.0;
  double filt_best = -2.0;  // best lower estimate so far of the largest eigenvalue below the locked cluster
  double filt_ref = 2.0;    // the Ritz value the planned filter is made large at
  double filt_rate = 0.0;   // growth exponent per degree of the planned filter at filt_ref
  double filt_lo = -1.0;    // lower end of the planned filter's damped interval
  // Estimate of the bottom of the spectrum of S, from below: the damped interval of the start-block filters is
  // [spec_lo, a] instead of [-1, a], which shortens the polynomial by a seventh to a fifth on kNN graphs (their
  // spectra end near -0.3 ... -0.5).  -1 until the first unfiltered steps have shown the smallest Ritz value (an upper
  // bound of the true bottom; after four block steps it was found 0.11 to 0.17 above it, so 0.25 is taken off); a
  // Ritz value seen near or below the estimate later lowers it.  An eigenvalue below the estimate is amplified instead
  // of damped - at worst as much as the wanted ones (x(-1) = -x(1) when the interval is symmetric about 0) -, which
  // costs block steps, never correctness: the phases converge by their own residual tests.
  double spec_lo = -1.0;
  bool spec_lo_set = false;
  bool late_off = false;    // projecting the locked vectors out after the filter has stopped paying (see run())
  int filt_extra = 0;       // degrees added to (or taken from) the planned degree: feedback from the phases' first steps
  sc_stats stats{};
  KTimer timer;

  double* rinv() { return small.p; }
  double* r1() { return small.p + kPP * kPP; }
  double* gram() { return small.p + 2 * kPP * kPP; }
  double* slot(int i) { return slots.p + (size_t)i * kSlotDoubles; }
  // scaling applied when the packed operand z of the next product is written: the CSR product scales by s on both
  // sides (z = s o x), the entry product has S multiplied out (z = x)
  const double* zs() const { return val_s.p ? nullptr : s.p; }
  double spmm_bytes() const {
    return 12.0 * (double)nnz + 8.0 * (double)(n + 1) + (val_s.p ? 0.0 : 8.0 * (double)n) + 16.0 * (double)n * b;
  }
  // y (row-major, leading dimension ldy) = S x for the block whose packed operand is in z
  void spmm_from_z(double* y, int64_t ldy) {
    if (val_s.p && resident.usable && resident.rest_row0 >= n && !no_resident_product) {
      // every diagonal block has work items of the LDS-resident form: a single product is that form's recurrence
      // with one step (u+ = 1 * (S u - 0 * u) - 0), read from LDS instead of gathered out of L2
      HIP_TRY(launch_cheb_resident(rowptr, col, val_s.p, z.p, y, ldy, b, 1, 1.0, 1.0, 0.0, resident.items.p,
                                   resident.nitems, resident.lds_bytes, resident.scol.p, resident.sval.p,
                                   resident.slice_base.p, resident.slice_len.p, st));
    } else if (val_s.p) {
      HIP_TRY(launch_spmm_vals(rowptr, col, val_s.p, n, z.p, b, y, ldy, avg_deg, longrows.p, nlong, st));
    } else {
      HIP_TRY(launch_spmm(rowptr, col, val, s.p, n, z.p, b, y, ldy, avg_deg, st));
    }
  }
  const double* hslot(int i) const { return slots_host.p + (size_t)i * kSlotDoubles; }

  void reorder() {
    rowptr_p.alloc((size_t)n + 1);
    col_p.alloc((size_t)nnz);
    val_p.alloc((size_t)nnz);
    old_of_new_d.alloc((size_t)n);
    new_of_old_d.alloc((size_t)n);
    // components too large for any item of the LDS-resident filter go last, as one run of rows that the filter leaves
    // to the product-per-step kernel (8-column items with two iterates: 128 bytes of LDS per row)
    int big_rows = 0;
    if ((b == 16 || b == 32) && !(flags & SC_FLAG_NO_START_FILTER)) big_rows = (device_lds_limit() - 1024) / 128;
    ncomp = reorder_csr(rowptr, col, val, n, nnz, rowptr_p.p, col_p.p, val_p.p, old_of_new_d.p, new_of_old_d.p,
                        (flags & SC_FLAG_COMPONENT_NULLSPACE) ? &comp_host : nullptr, b >= 8 ? 1 : 0, st, big_rows);
    rowptr = rowptr_p.p;
    col = col_p.p;
    val = val_p.p;
    rowmap = old_of_new_d.p;
    rowinv = new_of_old_d.p;
  }

  // Optional: the closed-form null vectors D^1/2 1_C / sqrt(vol C) of the first min(k, ncomp) components are
  // written into the basis and locked before any Lanczos phase (needs reorder()).
  void lock_component_nullspace() {
    const int take = std::min(k, ncomp);
    if (take <= 0) return;
    DevBuf<double> deg;
    deg.alloc((size_t)n);
    HIP_TRY(launch_degree_scaling(rowptr, val, n, deg.p, s.p, flag.p, st));
    std::vector<double> d((size_t)n), vol((size_t)ncomp, 0.0);
    HIP_TRY(hipMemcpyAsync(d.data(), deg.p, (size_t)n * sizeof(double), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    for (int64_t i = 0; i < n; ++i) vol[comp_host[i]] += d[i];
    for (int64_t i = 0; i < n; ++i) d[i] = std::sqrt(d[i] / vol[comp_host[i]]);
    comp_d.alloc((size_t)n);
    coef_d.alloc((size_t)n);
    HIP_TRY(hipMemcpyAsync(comp_d.p, comp_host.data(), (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(coef_d.p, d.data(), (size_t)n * sizeof(double), hipMemcpyHostToDevice, st));
    HIP_TRY(launch_nullspace_fill(basis.p, n, ld, 0, take, comp_d.p, coef_d.p, st));
    comp_d.release();
    coef_d.release();
    // Nothing is locked unverified: the residual S v - v of every vector is formed, b columns per product, and its
    // norm must meet tol like that of any Ritz pair (a component pass gone wrong, or a W that is not symmetric, shows
    // here).  If one fails, none is locked and the solve takes the plain path.
    std::vector<double> rho((size_t)take, 0.0), g((size_t)kPP * kPP);
    const int ycol = take + b;  // product block; columns [take, take + b) pad the last chunk with zeros
    HIP_TRY(hipMemsetAsync(z.p, 0, (size_t)n * b * sizeof(double), st));
    HIP_TRY(launch_copy_cols(z.p, b, 0, basis.p, ld, take, b, n, st));
    const ProjectPlan plan = plan_project(n, b, kMaxPartials);
    bool ok = true;
    for (int c0 = 0; c0 < take && ok; c0 += b) {
      const int w = std::min(b, take - c0);
      HIP_TRY(launch_pack_scaled(basis.p + c0, ld, zs(), n, b, z.p, st));
      spmm_from_z(basis.p + ycol, ld);
      HIP_TRY(launch_sub_cols(basis.p, ld, c0, basis.p, ld, ycol, w, n, st));
      HIP_TRY(launch_project(basis.p, n, ld, ycol, b, ycol, b, plan, part.p, st));
      HIP_TRY(launch_reduce_partials(part.p, plan.npart, b, b, gram(), nullptr, 0, nullptr, 0, st));
      HIP_TRY(hipMemcpyAsync(g.data(), gram(), g.size() * sizeof(double), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      stats.spmv_cols += w;
      for (int t = 0; t < w; ++t) {
        rho[c0 + t] = std::sqrt(std::max(g[(size_t)t * kPP + t], 0.0));
        if (!(rho[c0 + t] <= tol)) ok = false;
      }
    }
    if (!ok) {
      if (debug_on()) std::fprintf(stderr, "[sceig] component null vectors failed the residual test: plain path\n");
      return;
    }
    nl = take;
    theta_locked.assign(take, 1.0);
    rho_locked = rho;
  }

  void setup() {
    const double t0 = now_s();
    flag.alloc(1);
    HIP_TRY(hipMemsetAsync(flag.p, 0, sizeof(int), st));
    HIP_TRY(hipMemcpyAsync(&nnz, rowptr + n, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (nnz < 0) SC_THROW(SC_ECSR);
    HIP_TRY(launch_validate_csr(rowptr, col, n, nnz, flag.p, st));
    int hflag = 0;
    HIP_TRY(hipMemcpyAsync(&hflag, flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (hflag & 3) SC_THROW(SC_ECSR);
    if (ws_limit > 0) {  // a workspace that cannot hold the solve is refused before anything is computed
      sc_options o{};
      o.m = m;
      o.block = b;
      o.flags = flags;
      size_t need = 0;
      if (sc_workspace_bytes(n, nnz, k, &o, &need) != SC_OK || need > ws_limit) SC_THROW(SC_ENOMEM);
    }
    if (flags & SC_FLAG_VALIDATE_SYMMETRY) {
      HIP_TRY(launch_validate_symmetry(rowptr, col, val, n, flag.p, st));
      HIP_TRY(hipMemcpyAsync(&hflag, flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      if (hflag & (8 | 16)) SC_THROW(SC_ECSR);
    }
    const double t1 = now_s();
    if (!(flags & SC_FLAG_NO_REORDER)) reorder();
    const double t2 = now_s();
    s.alloc((size_t)n);
    HIP_TRY(launch_degree_scaling(rowptr, val, n, nullptr, s.p, flag.p, st));
    HIP_TRY(hipMemcpyAsync(&hflag, flag.p, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (hflag & 4) SC_THROW(SC_EZERODEG);
    avg_deg = (double)nnz / (double)n;
    if (b >= 8) {
      val_s.alloc((size_t)nnz);
      HIP_TRY(launch_scale_values(rowptr, col, val, s.p, val_s.p, n, st));
      // the rows the wide products hand to whole workgroups (hubs of the kNN graph)
      const size_t lw = long_row_list_workspace(n);
      DevBuf<char> lwork;
      DevBuf<int32_t> lcount;
      lwork.alloc(lw);
      lcount.alloc(1);
      longrows.alloc((size_t)n);
      HIP_TRY(long_row_list(rowptr, n, lwork.p, lw, longrows.p, lcount.p, st));
      int32_t hcount = 0;
      HIP_TRY(hipMemcpyAsync(&hcount, lcount.p, sizeof(int32_t), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      nlong = hcount;
      if (!(flags & SC_FLAG_NO_START_FILTER)) plan_resident(rowptr, col, val_s.p, n, nnz, b, st, &resident);
    }
    const double t3 = now_s();

    ld = ((int64_t)m + b + 15) / 16 * 16;
    basis.alloc((size_t)n * ld);
    z.alloc((size_t)n * b);
    const int jmax = m + b;
    part.alloc((size_t)kMaxPartials * jmax * kPP);
    gpart.alloc((size_t)kGramPartials * kPP * kPP);
    h1.alloc((size_t)jmax * kPP);
    hsum.alloc((size_t)jmax * kPP);
    small.alloc(3 * kPP * kPP);
    max_slots = m / b + 4;
    slots.alloc((size_t)max_slots * kSlotDoubles);
    slots_host.alloc((size_t)max_slots * kSlotDoubles);
    ystage.alloc(kYStageDoubles);
    rot_cols = (size_t)std::min(m, std::max(m / 2 + b, 2 * b));
    rot.alloc((size_t)n * rot_cols);
    yd_cap = (size_t)(m + b) * std::max<size_t>(rot_cols, (size_t)k);
    yd.alloc(yd_cap);
    perm_d.alloc((size_t)k);
    if ((flags & SC_FLAG_COMPONENT_NULLSPACE) && !(flags & SC_FLAG_NO_REORDER)) lock_component_nullspace();
    stats.components = ncomp;
    stats.t_setup = now_s() - t0;
    if (debug_on())
      std::fprintf(stderr, "[sceig] setup parts: validate %.0f us, reorder %.0f us, degrees+scaling %.0f us, buffers %.0f us\n",
                   (t1 - t0) * 1e6, (t2 - t1) * 1e6, (t3 - t2) * 1e6, (now_s() - t3) * 1e6);
    if (debug_on()) std::fprintf(stderr, "[sceig] setup %.3fs: n=%lld nnz=%lld components=%d m=%d b=%d locked=%d\n",
                                 stats.t_setup, (long long)n, (long long)nnz, ncomp, m, b, nl);
  }

  // ---- one block step on the last active block (columns [nl+ja-b, nl+ja)), results into slot si
  // tentative: the new block is orthogonalized against the active Krylov columns only, not against the locked
  // vectors.  Its residual estimates then still contain what the product holds along the locked vectors, so they
  // are upper bounds of the proper ones: pairs that pass the test with them are converged, and the Ritz vectors
  // (combinations of the active columns, which are orthogonal to the locked vectors) are unaffected.  The first
  // step after a filtered start block is taken this way - most phases end with it, and the pass over all locked
  // vectors, the most expensive thing a step does once many are locked, is never made for them; if the test fails
  // the step is taken again in full.
  void enqueue_step(int ja, int si, bool tentative = false) {
    const int jt = nl + ja;
    timer.begin(kFamSpmm);
    spmm_from_z(basis.p + jt, ld);
    timer.end(kFamSpmm, spmm_bytes(), 2.0 * (double)nnz * b);
    double* sl = slot(si);
    // A tentative step makes one Gram-Schmidt pass, not two: its block never joins the basis, so the orthogonality a
    // second pass would restore is not needed, and the residual block W - V (V^T W) itself comes out of one pass to
    // rounding relative to W (1e-16 of a block of norm one, against residuals of the size of tol).
    const bool one_pass = tentative && !tentative_two_passes;
    const int ngram = enqueue_cgs2(basis.p, n, ld, jt, jt, b, one_pass ? jt : nl, part.p, h1.p, hsum.p, sl, jt - b, gpart.p,
                                   st, &timer, tentative ? nl : 0, one_pass && b < kWideUpdate);
    if (tentative && ngram > 0) {
      // Only the Gram matrix of the residual block is looked at (residual estimates; a block that vanished): the
      // block is not orthonormalized, since it either is dropped with the phase or built again.  The slot of the QR
      // factor gets the Gram matrix too: its diagonal vanishes exactly when the factor's would.
      timer.begin(kFamQr);
      HIP_TRY(launch_reduce_partials(gpart.p, ngram, b, b, sl + 2 * kPP * kPP, nullptr, 0, nullptr, 0, st));
      HIP_TRY(launch_reduce_partials(gpart.p, ngram, b, b, sl + kPP * kPP, nullptr, 0, nullptr, 0, st));
      timer.end(kFamQr, 0.0, 0.0);
    } else {
      enqueue_block_qr(basis.p, n, ld, jt, b, part.p, gpart.p, ngram, gram(), rinv(), r1(), sl + kPP * kPP,
                       sl + 2 * kPP * kPP, z.p, zs(), st, &timer);
    }
    stats.block_steps += 1;
    stats.spmv_cols += b;
  }

  void fetch_slots(int first, int count) {
    if (count <= 0) return;
    HIP_TRY(hipMemcpyAsync(slots_host.p + (size_t)first * kSlotDoubles, slots.p + (size_t)first * kSlotDoubles,
                           (size_t)count * kSlotDoubles * sizeof(double), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    ystage_busy = false;
  }

  // Start-block filter.  The block at columns [nl, nl+b) (orthonormal, its s-scaled packed copy in z) is replaced
  // by p(S) applied to it, p = Chebyshev polynomial of degree d of the interval [-1, a] mapped to [-1, 1]: what lies
  // in [-1, a] stays bounded by 1, what lies above a grows like cosh(d acosh(x)).  Only products and a three-term
  // recurrence: no reorthogonalization.  The caller orthogonalizes and orthonormalizes the result again.
  // rnd_key / use_rnd: the block to filter is random block rnd_key, which the one-launch form makes in its prologue
  // (the caller has checked that this form takes every row); z is then not read
  void apply_start_filter(int d, double a, uint64_t rnd_key = 0, int use_rnd = 0) {
    double* buf1 = rot.p;
    double* buf2 = rot.p + (size_t)n * b;
    double* buf3 = rot.p + 2 * (size_t)n * b;
    if (!val_s.p) HIP_TRY(launch_copy_cols(basis.p, ld, nl, buf1, b, 0, b, n, st));
    // double-precision steps at the end: as many as damp the unwanted directions by 2,000 against the wanted ones at
    // the planned growth per degree (single-precision rounding, 6e-8, then ends below 1e-10), and at least six
    int tail = filter_tail64;
    if (filt_rate > 0.0) tail = std::max(tail, (int)std::ceil(std::log(2000.0) / filt_rate));
    int d32 = d > tail + 1 ? d - tail : 0;
    {
      // no single-precision step may overflow: the polynomial grows fastest at an end of the spectrum, +1 or (when
      // the damped interval starts too high) -1; the start block's entries are at most 1, float reaches 3e38
      const double lo = filt_lo;
      const double xm = std::max(std::fabs((-2.0 - a - lo) / (a - lo)), std::fabs((2.0 - a - lo) / (a - lo)));
      const double growth = xm > 1.0 ? std::acosh(xm) : 0.0;
      if (growth > 0.0) d32 = std::min(d32, (int)std::floor(69.0 / growth));  // e^69 = 1e30
      if (d32 < 1) d32 = 0;
    }
    const double* res = enqueue_cheb_filter(rowptr, col, val, val_s.p, s.p, n, nnz, b, d, a, z.p, buf1, buf2, buf3,
                                            avg_deg, longrows.p, nlong, &resident, st, &timer, basis.p + nl, ld, filt_lo,
                                            d32, rnd_key, use_rnd);
    stats.spmv_cols += (int64_t)d * b;
    stats.filter_steps += d;
    if (res) HIP_TRY(launch_copy_cols(res, b, 0, basis.p, ld, nl, b, n, st));
  }

  // Decide the filter of the next start block from the Ritz values theta (ascending, ghosts at the bottom).
  //
  // locked = true: a phase has just locked its `nlead` leading pairs.  Further copies of the locked eigenvalues may
  // remain (a block Krylov space holds at most b of them), so the polynomial is made large at the smallest value
  // just locked and small below an estimate `a` of what follows: the largest unlocked Ritz value when a gap
  // separates it from the locked ones (it approaches the next distinct eigenvalue from below; the best such
  // estimate over the phases is kept, and reused when a phase has no unlocked Ritz value to offer), otherwise the
  // larger of that kept estimate and the (b+1)-th unlocked one, below the b values the next phase is after.
  // locked = false: a phase that started unfiltered looks at its first Ritz values; nothing has converged, the
  // target is the largest Ritz value and `a` the kept estimate if there is one, else the (nlead+1)-th Ritz value.
  //
  // A filter that is not worth its products (amplification below 100 at the degree cap) is left out.  A wrong guess
  // costs convergence speed, never correctness: the Lanczos phase that follows converges by its own residual test.
  void plan_start_filter(const std::vector<double>& theta, int ja, int nlead, int nghost, bool locked) {
    filt_d = 0;
    if (flags & SC_FLAG_NO_START_FILTER) return;
    if (rot_cols < (size_t)3 * b) return;
    if (nlead < 1 || ja - nghost < nlead) return;
    const int nu = ja - nlead - nghost;  // Ritz values of real directions below the leading ones
    const double th_ref = locked ? theta[ja - nlead] : theta[ja - 1];
    if (filt_best >= th_ref - 1e-6) filt_best = -2.0;  // the wanted values have moved below the old estimate
    double a = filt_best;
    if (locked && nu >= 1) {
      const double u1 = theta[ja - 1 - nlead];
      const double ub = theta[std::max(ja - 1 - nlead - b, nghost)];
      if (th_ref - u1 > u1 - ub) {
        filt_best = std::max(filt_best, u1);
        a = filt_best;
      } else {
        a = std::max(ub, filt_best);  // an estimate kept from a phase that did see a gap outranks a Ritz value far below it
      }
    } else if (!locked && filt_best <= -2.0 && nu >= 1) {
      a = theta[ja - 1 - nlead];
    }
    const double lo = spec_lo;
    if (!(a > lo + 0.05) || !(a < th_ref)) return;
    a += 0.03 * (th_ref - a);  // Ritz values approach the eigenvalue they estimate from below
    const double xt = (2.0 * th_ref - a - lo) / (a - lo);
    const double rate = std::acosh(xt);
    // what lies below `a` should end up near tol relative to the wanted directions, so that the Lanczos steps
    // after the filter mostly confirm convergence
    const double amp = std::min(1e12, std::max(1e6, 100.0 / std::max(tol, 1e-300)));
    const int dmax = 30;
    if (!(rate > 0.0) || std::cosh(dmax * rate) < 100.0) return;
    const int d = (int)std::ceil(std::log(2.0 * amp) / rate) + filt_extra;
    filt_d = std::min(std::max(d, 2), dmax);
    filt_a = a;
    filt_lo = lo;
    filt_ref = th_ref;
    filt_rate = rate;
  }

  // basis[:, dst : dst+l] = basis[:, nl : nl+ja] * Y[:, sel] (through the rotation workspace when l > 64)
  void rotate_into(int ja, const std::vector<double>& ymat, int ycols, const std::vector<int>& sel, int dst) {
    const int l = (int)sel.size();
    if (l == 0) return;
    if ((size_t)ja * l > yd_cap || (size_t)l > rot_cols) SC_THROW(SC_EDOMAIN);
    const size_t count = (size_t)ja * l;
    const bool staged = count <= kYStageDoubles;  // small blocks go through pinned memory: nothing to wait for
    std::vector<double> ybig;
    if (staged && ystage_busy) {
      HIP_TRY(hipStreamSynchronize(st));
      ystage_busy = false;
    }
    if (!staged) ybig.resize(count);
    double* yl = staged ? ystage.p : ybig.data();
    for (int r = 0; r < ja; ++r)
      for (int t = 0; t < l; ++t) yl[(size_t)r * l + t] = ymat[(size_t)r * ycols + sel[t]];
    HIP_TRY(hipMemcpyAsync(yd.p, yl, count * sizeof(double), hipMemcpyHostToDevice, st));
    timer.begin(kFamRotate);
    if (l <= 64) {
      // one wave holds all l results of a row before it stores any: straight into the basis, also over its own inputs
      HIP_TRY(launch_row_gemm(basis.p, n, ld, nl, ja, yd.p, l, l, 3, dst, nullptr, 0, nullptr, st));
    } else {
      HIP_TRY(launch_row_gemm(basis.p, n, ld, nl, ja, yd.p, l, l, 1, 0, rot.p, l, nullptr, st));
    }
    timer.end(kFamRotate, 8.0 * (double)n * (ja + l), 2.0 * (double)n * ja * l);
    if (l > 64) HIP_TRY(launch_copy_cols(rot.p, l, 0, basis.p, ld, dst, l, n, st));
    if (staged)
      ystage_busy = true;
    else
      HIP_TRY(hipStreamSynchronize(st));  // ybig (pageable host memory) must stay alive until the copy is done
  }

  // drop locked column `idx` by moving the last locked column into its place
  void drop_locked(int idx) {
    const int last = nl - 1;
    if (idx != last) {
      HIP_TRY(launch_copy_cols(basis.p, ld, last, rot.p, 1, 0, 1, n, st));
      HIP_TRY(launch_copy_cols(rot.p, 1, 0, basis.p, ld, idx, 1, n, st));
      theta_locked[idx] = theta_locked[last];
      rho_locked[idx] = rho_locked[last];
    }
    theta_locked.pop_back();
    rho_locked.pop_back();
    nl -= 1;
  }

  double kth_locked_theta() const {
    std::vector<double> t(theta_locked);
    std::sort(t.begin(), t.end(), std::greater<double>());
    return t[k - 1];
  }

  int run(double* evals_out, double* evecs_out) {
    const double t_begin = now_s();
    timer.st = st;
    setup();
    int cycles = 0;
    bool not_converged = false;
    bool finished = false;
    int prev_phase_steps = 0, prev_filtered_steps = 0;
    uint64_t stream_id = 0;

    ProjectedMatrix T;
    T.init(m);
    std::vector<double> Tsub, Y;
    SelectedEig seig;
    int ycols = 0;
    std::vector<char> ghost;

    while (!finished) {
      const bool verifying = nl >= k;
      if (verifying && (flags & SC_FLAG_NO_VERIFY)) break;
      // W >= 0 makes D^-1 W row-stochastic, so no eigenvalue of S exceeds 1: once the k-th locked theta is within
      // tol of 1 a check phase could not find anything better by more than tol
      if (verifying && kth_locked_theta() + tol >= 1.0) break;
      if ((int64_t)nl >= n) break;
      const bool last_cycle_phase = cycles >= maxiter;  // out of budget: only build enough Ritz vectors to answer
      if (last_cycle_phase && verifying) {
        break;  // k pairs are locked, the check phase could not be afforded
      }
      const int cap = m - nl;  // active columns allowed (excluding the block under construction)
      const int want = verifying ? 1 : std::min(b, k - nl);
      cycles += last_cycle_phase ? 0 : 1;
      stats.phases += 1;

      // ---- start block
      bool filtered = filt_d > 0;
      // exponent of the filter this phase starts from (0: none, or not a random block), for the degree feedback
      double phase_rate = filtered ? filt_rate : 0.0;
      // The locked vectors' eigenvalues lie above the damped interval too, so the filter amplifies what a block holds
      // along them.  When none of them lies above the value the filter is aimed at (the usual case here: further
      // copies of one multiple eigenvalue), they are amplified no more than the wanted directions, the filtered block
      // keeps a fair share of its norm outside their span, and projecting them out AFTER the filter loses nothing to
      // cancellation: the random block goes into the filter as it is, and one Gram-Schmidt pass afterwards - a second
      // only if the device-side test asks for it - takes the place of a pass before and a pass after the filter.
      // Otherwise (locked eigenvalues above the target: they would swamp the block) the block is projected first.
      bool late_projection = false;
      // The price of projecting afterwards: the locked vectors x_i are eigenvectors only to within their residuals, so
      // removing span(X) from the amplified block leaves, of what it held along the exact eigenvectors behind X, a
      // part of relative size (angle between the two spans) * sqrt(locked / remaining directions), made of unwanted
      // eigenvectors.  That floor under the first step's residuals grows as the wanted directions run out; once a
      // phase sees it near tol (late_off) the later phases project before the filter again.
      if (filtered && nl > 0 && !no_late_projection && !late_off) {
        const double top = *std::max_element(theta_locked.begin(), theta_locked.end());
        late_projection = top <= filt_ref + 1e-6;
      }
      // the random block; when it goes into the filter as it is (the wide blocks' operand is a plain packed copy) it is
      // drawn into the packed buffer directly: same numbers, one pass less
      const bool use_v0 = v0 && stats.phases == 1;
      const bool random_packed = filtered && late_projection && val_s.p && !use_v0;
      // ... and where the one-launch filter takes every row it makes those numbers itself: no pass to write them
      const bool random_inside = random_packed && resident.usable && resident.rest_row0 >= n && !no_random_inside;
      uint64_t rnd_key = 0;
      if (random_inside) {
        rnd_key = random_block_key(seed, stream_id++);
      } else if (random_packed) {
        HIP_TRY(launch_random_block(z.p, n, b, 0, b, seed, stream_id++, st));
      } else {
        HIP_TRY(launch_random_block(basis.p, n, ld, nl, b, seed, stream_id++, st));
        if (use_v0)  // the caller's start vector leads the first block, the other columns stay random
          HIP_TRY(launch_set_column(basis.p, n, ld, nl, v0, rowmap, st));
      }
      if (filtered) {
        if (debug_on())
          std::fprintf(stderr, "[sceig] t=%.4fs phase %d start block filtered: degree %d, damped interval [%.4f, %.6f]%s\n",
                       now_s() - t_begin, stats.phases, filt_d, filt_lo, filt_a,
                       late_projection ? ", locked vectors projected out afterwards" : "");
        if (!late_projection)
          (void)enqueue_cgs2(basis.p, n, ld, nl, nl, b, nl, part.p, h1.p, hsum.p, nullptr, 0, nullptr, st, &timer);
        if (!random_packed) HIP_TRY(launch_pack_scaled(basis.p + nl, ld, zs(), n, b, z.p, st));
        apply_start_filter(filt_d, filt_a, rnd_key, random_inside ? 1 : 0);
        filt_d = 0;
      }
      // a block that went into the filter orthogonal to the locked vectors picked up along them since only what is of
      // the order of their residuals relative to the block, so one projection removes it without cancellation
      const int ngram0 =
          late_projection
              ? enqueue_cgs_adaptive(basis.p, n, ld, nl, nl, b, part.p, h1.p, hsum.p, gpart.p, gram(), flag.p, st, &timer)
              : enqueue_cgs2(basis.p, n, ld, nl, nl, b, filtered ? nl : 0, part.p, h1.p, hsum.p, nullptr, 0, gpart.p, st,
                             &timer);
      enqueue_block_qr(basis.p, n, ld, nl, b, part.p, gpart.p, ngram0, gram(), rinv(), r1(), slot(0) + kPP * kPP,
                       slot(0) + 2 * kPP * kPP, z.p, zs(), st, &timer);
      int ja = b;            // active columns whose coupling is (or will be) assembled
      int assembled = 0;     // active columns of T that are final (their block has been multiplied by S)
      int next_slot = 1;     // slot 0 = start block QR
      int fetched = 0;       // slots already on the host
      int steps_in_phase = 0;
      T.clear();
      ghost.assign((size_t)cap + b, 0);
      bool start_block_seen = false;
      int pending = 0;
      const int prev_steps = filtered ? prev_filtered_steps : prev_phase_steps;
      int next_check = prev_steps > 1 ? prev_steps - 1 : (filtered ? 1 : 4);
      double last_rho = -1.0;
      int last_rho_step = 0;
      bool phase_over = false;
      // Block steps until the next inspection, from the decay of the residual estimate r_now of the last wanted pair
      // since the previous inspection of this phase: 85 % of the steps that rate needs to reach tol, at most 12 -
      // unless that is more than twice the `room` steps left before the basis is full (Lanczos converges faster
      // than its early rate, hence the factor), when only the restart inspects.
      auto schedule_check = [&](double r_now, int room) {
        int next = std::max(1, check_every);
        if (last_rho > 0.0 && r_now > 0.0 && r_now < last_rho && steps_in_phase > last_rho_step) {
          const double rate = std::log(last_rho / r_now) / (steps_in_phase - last_rho_step);
          const double need = std::log(r_now / std::max(tol, 1e-300)) / rate;
          const int guess = (int)std::floor(0.85 * std::min(need, 1e6));
          next = guess > 2 * room ? room + 1 : std::min(std::max(guess, 1), 12);
        }
        last_rho = r_now;
        last_rho_step = steps_in_phase;
        return next;
      };

      // worth it only where the pass over the locked vectors costs more than a repeated step does when the test
      // fails (a product, two passes over the start block and its QR): from about 2e7 locked entries on
      bool tentative_allowed = filtered && nl > 0 && !last_cycle_phase && !no_tentative_step &&
                               (double)n * nl >= tentative_min_work;
      // The floor under a late projection's residuals ends near sqrt(locked / remaining wanted directions) times the
      // locked residuals.  The multiplicity of the eigenvalue 1 of S is the number of connected components, which the
      // renumbering has counted: when k asks for (nearly) all of them the ratio gets large.  A hint for the degree
      // feedback only.
      const bool tight_target =
          tentative_allowed && ncomp > 0 && (double)(k - b) > 4.0 * std::max(ncomp - (k - b), 1);
      if (tentative_allowed) next_check = 1;  // a look after the cheap first step costs far less than a full second step
      while (!phase_over) {
        if (next_slot >= max_slots) SC_THROW(SC_EDOMAIN);  // cannot happen: a cycle has at most m/b steps
        // the phase's first step, inspected right after it, with room for its block in the basis
        const bool tentative = tentative_allowed && steps_in_phase == 0 && ja == b && next_check <= 1 && ja + b <= cap;
        enqueue_step(ja, next_slot, tentative);
        ++next_slot;
        ++pending;
        ++steps_in_phase;
        const bool full = ja + b > cap;  // the block just built cannot join the active basis
        bool check = full || pending >= next_check;
        if (last_cycle_phase && !verifying && ja >= std::min(k - nl, cap - b)) check = true;
        if (!check) {
          ja += b;
          continue;
        }
        // ---- inspect: bring the slots over and assemble T
        T.touch(ja + b);
        fetch_slots(fetched, next_slot - fetched);
        fetched = next_slot;
        if (!start_block_seen) {
          const double* r0 = hslot(0) + kPP * kPP;
          for (int x = 0; x < b; ++x) ghost[x] = (r0[x * kPP + x] == 0.0);
          start_block_seen = true;
        }
        // steps (next_slot - pending) .. (next_slot - 1); step with slot q worked on the block that
        // ends at active column  e_q = ja - (next_slot - 1 - q) * b
        for (int q = next_slot - pending; q < next_slot; ++q) {
          const int e = ja - (next_slot - 1 - q) * b;
          const int c0 = e - b;
          const double* A = hslot(q);
          for (int x = 0; x < b; ++x)
            for (int y = 0; y < b; ++y)
              T.at(c0 + x, c0 + y) = 0.5 * (A[x * kPP + y] + A[y * kPP + x]);
          for (int x = 0; x < b; ++x)
            if (ghost[c0 + x]) {
              for (int y = 0; y < e; ++y) T.at(c0 + x, y) = T.at(y, c0 + x) = 0.0;
              T.at(c0 + x, c0 + x) = -2.0;
            }
          assembled = e;
          if (q + 1 < next_slot) {
            // the block built by step q joined the basis: coupling R and ghost flags
            const double* R = hslot(q) + kPP * kPP;
            for (int x = 0; x < b; ++x) {
              ghost[e + x] = (R[x * kPP + x] == 0.0);
              for (int y = 0; y < b; ++y) {
                T.at(e + x, c0 + y) = R[x * kPP + y];
                T.at(c0 + y, e + x) = R[x * kPP + y];
              }
            }
          }
        }
        pending = 0;
        // ---- Ritz pairs of T[0:ja, 0:ja]: all values, vectors only for the leading ones that may be used
        const double te0 = now_s();
        Tsub.resize((size_t)ja * ja);
        for (int x = 0; x < ja; ++x) std::memcpy(&Tsub[(size_t)x * ja], &T.at(x, 0), sizeof(double) * ja);
        if (seig.factor(Tsub.data(), ja) != 0) SC_THROW(SC_EHIP);
        const std::vector<double>& theta = seig.values();
        const double* Rl = hslot(next_slot - 1) + kPP * kPP;
        const double* Gl = hslot(next_slot - 1) + 2 * kPP * kPP;
        int nreal = 0;
        for (int x = 0; x < ja; ++x) nreal += ghost[x] ? 0 : 1;
        bool exhausted = true;
        for (int x = 0; x < b; ++x) exhausted = exhausted && (Rl[x * kPP + x] == 0.0);
        // thick-restart size, should this inspection end in a restart
        int l_restart = std::max(want + b, ja / 2);
        l_restart = std::min({l_restart, ja - b, nreal, (int)rot_cols});
        int nsel = std::min(nreal, std::max(b, full ? l_restart : 0));
        auto ritz_vectors = [&](int count) {  // Y: ja x count, column t = Ritz vector of the t-th largest theta
          std::vector<int> idx(count);
          for (int t = 0; t < count; ++t) idx[t] = ja - 1 - t;
          Y.resize((size_t)ja * std::max(count, 1));
          seig.vectors(idx.data(), count, Y.data());
          ycols = count;
        };
        ritz_vectors(nsel);
        stats.t_host_eig += now_s() - te0;
        stats.host_eigs += 1;
        // residual estimates of the leading pairs (ghosts sit at -2, i.e. at the bottom of the spectrum)
        std::vector<double> rho(nsel);
        for (int t = 0; t < nsel; ++t) {
          double acc = 0.0;
          for (int x = 0; x < b; ++x) {
            double gx = 0.0;
            for (int y = 0; y < b; ++y) gx += Gl[x * kPP + y] * Y[(size_t)(ja - b + y) * ycols + t];
            acc += gx * Y[(size_t)(ja - b + x) * ycols + t];
          }
          rho[t] = std::sqrt(std::max(acc, 0.0));
        }
        int lead = 0;
        while (lead < nsel && rho[lead] <= tol) ++lead;
        if (nreal > 0 && spec_lo > -1.0 && theta[ja - nreal] < spec_lo + 0.02) {
          // a Ritz value at or below the assumed bottom of the spectrum: the filters have been amplifying there
          spec_lo = std::max(-1.0, theta[ja - nreal] - 0.1);
          if (debug_on())
            std::fprintf(stderr, "[sceig] t=%.4fs spectrum bottom estimate lowered to %.4f\n", now_s() - t_begin, spec_lo);
        }
        if (phase_rate > 0.0 && steps_in_phase == 1) {
          // Degree feedback.  How much of a filtered random block lies along the wanted directions shrinks as fewer of
          // them remain, so the same polynomial leaves relatively more of the rest: aim the first step's worst wanted
          // residual estimate at a target by adding the degrees the miss is worth (or giving one back when the filter
          // overshoots by more than a degree and a half).  The target is tol / 8, except where the floor described at
          // the phase start would otherwise reach tol before the end: it is proportional to the residuals the vectors
          // were locked with, so tol / 100 (two or three more degrees) keeps it down.  That is bought only where the
          // passes over the locked vectors are what a phase costs (tight_target).  With the wider target a miss of half
          // a degree already counts: tol / 8 less one degree (a factor 3 to 4) is within the spread between the columns
          // of one block, and a pair that misses tol costs two further block steps, a degree one product.
          double rw = 0.0;
          for (int t = 0; t < std::min(want, nsel); ++t) rw = std::max(rw, rho[t]);
          if (rw > 0.0) {
            const double target = (late_projection && tight_target ? 0.01 : 0.125) * tol;
            const double need = std::log(rw / target) / phase_rate;
            if (late_projection && rw > 0.5 * tol)
              late_off = true;  // the floor, not the polynomial: more degrees would not help
            else if (need > (late_projection && tight_target ? 1.0 : 0.5))  // see above
              filt_extra = std::min(filt_extra + (int)std::ceil(need), 6);
            else if (need < -1.5)
              filt_extra = std::max(filt_extra - 1, -4);
          }
          phase_rate = 0.0;  // once per phase
        }
        if (debug_on()) {
          const int wi = std::min(want, nsel) - 1;
          std::fprintf(stderr,
                       "[sceig] t=%.4fs phase %d step %d nl=%d ja=%d cap=%d full=%d lead=%d/%d theta[0]=%.12f rho[0]=%.2e "
                       "theta[w]=%.12f rho[w]=%.2e\n",
                       now_s() - t_begin, stats.phases, steps_in_phase, nl, ja, cap, (int)full, lead, want,
                       theta[ja - 1], rho[0], wi >= 0 ? theta[ja - 1 - wi] : 0.0, wi >= 0 ? rho[wi] : 0.0);
        }

        if (tentative && !(lead >= want || exhausted)) {
          // the upper bounds did not pass: the step again, this time with the projection against the locked vectors
          if (debug_on())
            std::fprintf(stderr, "[sceig] t=%.4fs phase %d first step repeated in full\n", now_s() - t_begin, stats.phases);
          HIP_TRY(launch_pack_scaled(basis.p + nl, ld, zs(), n, b, z.p, st));  // the product's operand: the start block
          tentative_allowed = false;
          ja = b;
          assembled = 0;
          next_slot = 1;
          fetched = 1;  // slot 0 (the start block's QR) is on the host already
          pending = 0;
          steps_in_phase = 0;
          T.clear();
          std::fill(ghost.begin() + b, ghost.end(), 0);
          next_check = 1;
          last_rho = -1.0;
          last_rho_step = 0;
          continue;
        }
        if (nreal == 0) {  // the deflated space is empty: nothing more exists
          finished = true;
          if (nl < k) not_converged = true;
          break;
        }
        if (!filtered && !full && !last_cycle_phase && !exhausted && lead < want && steps_in_phase >= 4 && nsel >= b) {
          // A phase that began from a plain random block (no spectrum estimate was available then): once its Ritz
          // values give one, filter the leading Ritz vectors - a far better start than a random block - and begin
          // the phase anew from the filtered block.
          if (debug_on())
            std::fprintf(stderr, "[sceig] smallest Ritz values after %d unfiltered steps: %.4f %.4f %.4f (ghosts %d)\n",
                         steps_in_phase, theta[ja - nreal], theta[std::min(ja - 1, ja - nreal + 1)],
                         theta[std::min(ja - 1, ja - nreal + 2)], ja - nreal);
          if (nreal > 0 && !no_spectrum_bottom && !spec_lo_set) {  // once: later Ritz values can only lower it
            spec_lo = std::max(-1.0, theta[ja - nreal] - 0.25);
            if (const char* forced = std::getenv("SCEIG_SPECTRUM_BOTTOM"))  // for tests of a wrong estimate
              spec_lo = std::min(0.9, std::max(-1.0, std::atof(forced)));
            spec_lo_set = true;
          }
          plan_start_filter(theta, ja, std::min(want, nreal), ja - nreal, false);
          if (filt_d > 0) {
            if (debug_on())
              std::fprintf(stderr, "[sceig] t=%.4fs phase %d restarts from its %d leading Ritz vectors filtered: degree %d, "
                           "damped interval [%.4f, %.6f]\n", now_s() - t_begin, stats.phases, b, filt_d, filt_lo, filt_a);
            std::vector<int> sel(b);
            for (int t = 0; t < b; ++t) sel[t] = t;
            rotate_into(ja, Y, ycols, sel, nl);
            HIP_TRY(launch_pack_scaled(basis.p + nl, ld, zs(), n, b, z.p, st));
            apply_start_filter(filt_d, filt_a);
            const int ngram1 = enqueue_cgs2(basis.p, n, ld, nl, nl, b, nl, part.p, h1.p, hsum.p, nullptr, 0, gpart.p, st, &timer);
            enqueue_block_qr(basis.p, n, ld, nl, b, part.p, gpart.p, ngram1, gram(), rinv(), r1(), slot(0) + kPP * kPP,
                             slot(0) + 2 * kPP * kPP, z.p, zs(), st, &timer);
            filt_d = 0;
            filtered = true;
            ja = b;
            assembled = 0;
            next_slot = 1;
            fetched = 0;
            steps_in_phase = 0;
            T.clear();
            std::fill(ghost.begin(), ghost.end(), 0);
            start_block_seen = false;
            next_check = prev_filtered_steps > 1 ? prev_filtered_steps - 1 : 1;
            last_rho = -1.0;
            last_rho_step = 0;
            continue;
          }
        }
        const bool stop_now = last_cycle_phase && !verifying;
        if ((lead >= want || exhausted) && !stop_now) {
          int nlock = std::min(lead, verifying ? b : want);
          if (exhausted && nlock == 0) nlock = std::min(nreal, want);
          if (verifying) {
            const double kth = kth_locked_theta();
            int better = 0;
            while (better < nlock && theta[ja - 1 - better] > kth + tol) ++better;
            nlock = better;
            if (nlock == 0) {
              finished = true;
              break;
            }
          }
          std::vector<int> sel(nlock);
          for (int t = 0; t < nlock; ++t) sel[t] = t;
          rotate_into(ja, Y, ycols, sel, nl);
          for (int t = 0; t < nlock; ++t) {
            theta_locked.push_back(theta[ja - 1 - t]);
            rho_locked.push_back(rho[t]);
          }
          nl += nlock;
          while (nl > k) {  // keep the k best
            int worst = 0;
            for (int t = 1; t < nl; ++t)
              if (theta_locked[t] < theta_locked[worst]) worst = t;
            drop_locked(worst);
          }
          phase_over = true;
          (filtered ? prev_filtered_steps : prev_phase_steps) = steps_in_phase;
          plan_start_filter(theta, ja, nlock, ja - nreal, true);
          break;
        }
        if (stop_now || (full && cycles >= maxiter)) {
          // out of cycles: take the best unconverged Ritz vectors to fill up the answer
          const int take = std::min({nreal, std::max(0, k - nl), (int)rot_cols});
          if (take > nsel) ritz_vectors(take);
          std::vector<int> sel(take);
          for (int t = 0; t < take; ++t) sel[t] = t;
          rotate_into(ja, Y, ycols, sel, nl);
          for (int t = 0; t < take; ++t) {
            theta_locked.push_back(theta[ja - 1 - t]);
            rho_locked.push_back(t < nsel ? rho[t] : 1.0);
          }
          nl += take;
          not_converged = true;
          finished = true;
          break;
        }
        if (full) {
          // ---- thick restart: keep the leading Ritz vectors and the residual block
          cycles += 1;
          stats.restarts += 1;
          const int l = l_restart;
          if (l < 1) SC_THROW(SC_EDOMAIN);
          if (l > ycols) ritz_vectors(l);
          std::vector<int> sel(l);
          for (int t = 0; t < l; ++t) sel[t] = t;
          rotate_into(ja, Y, ycols, sel, nl);
          HIP_TRY(launch_copy_cols(basis.p, ld, nl + ja, rot.p, b, 0, b, n, st));
          HIP_TRY(launch_copy_cols(rot.p, b, 0, basis.p, ld, nl + l, b, n, st));
          T.clear();
          T.touch(l + b);
          std::fill(ghost.begin(), ghost.end(), 0);
          for (int t = 0; t < l; ++t) T.at(t, t) = theta[ja - 1 - t];
          for (int x = 0; x < b; ++x) {
            ghost[l + x] = (Rl[x * kPP + x] == 0.0);
            for (int t = 0; t < l; ++t) {
              double c = 0.0;
              for (int y = 0; y < b; ++y) c += Rl[x * kPP + y] * Y[(size_t)(ja - b + y) * ycols + t];
              T.at(l + x, t) = c;
              T.at(t, l + x) = c;
            }
          }
          ja = l + b;
          assembled = l;
          next_slot = 1;
          fetched = 1;
          // The residual of the last wanted pair keeps decaying across restarts: when the rate observed so far says
          // that convergence is further away than the basis has room for, the next inspection worth its projected
          // eigenproblem is the one at the next restart.
          next_check = schedule_check(rho[std::min({want, nreal, nsel}) - 1], (cap - ja) / b + 1);
          continue;
        }
        // ---- continue: the new block joins; schedule the next inspection from the observed decay
        {
          const double* R = Rl;
          const int e = ja, c0 = ja - b;
          for (int x = 0; x < b; ++x) {
            ghost[e + x] = (R[x * kPP + x] == 0.0);
            for (int y = 0; y < b; ++y) {
              T.at(e + x, c0 + y) = R[x * kPP + y];
              T.at(c0 + y, e + x) = R[x * kPP + y];
            }
          }
          ja += b;
          next_check = schedule_check(rho[std::min({want, nreal, nsel}) - 1], (cap - ja) / b + 1);
        }
        (void)assembled;
      }
    }

    // ---- outputs.  Every locked vector is a Ritz vector whose residual estimate met tol (and theta its Rayleigh
    // quotient), the locked set is orthonormal by construction, so the answer is the locked set in descending
    // order of theta.  A Rayleigh-Ritz step over the locked vectors (the Ritz-vector step of Algorithm 3 applied
    // to the final basis) is added when some vector did not converge, or on request.
    const int nx = nl;
    bool all_converged = !not_converged;
    for (size_t t = 0; t < rho_locked.size(); ++t) all_converged = all_converged && rho_locked[t] <= tol;
    const bool final_rr = !all_converged || (flags & SC_FLAG_FINAL_RR);
    if (debug_on())
      std::fprintf(stderr, "[sceig] t=%.4fs %s over %d locked vectors\n", now_s() - t_begin,
                   final_rr ? "Rayleigh-Ritz" : "sorted output", nx);
    std::vector<double> evals_host(k_out, std::numeric_limits<double>::quiet_NaN());
    int nfound = std::min(nx, k_out);
    if (nx < k_out) HIP_TRY(hipMemsetAsync(evecs_out, 0, (size_t)n * k_out * sizeof(double), st));
    std::vector<int32_t> order;
    if (nx > 0 && !final_rr) {
      order.resize(nx);
      std::iota(order.begin(), order.end(), 0);
      std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return theta_locked[x] > theta_locked[y]; });
      order.resize(nfound);
      for (int t = 0; t < nfound; ++t) evals_host[t] = 1.0 - theta_locked[order[t]];
      std::vector<int32_t> outpos((size_t)nx, -1);  // output column of every locked basis column
      for (int t = 0; t < nfound; ++t) outpos[order[t]] = t;
      HIP_TRY(hipMemcpyAsync(perm_d.p, outpos.data(), (size_t)nx * sizeof(int32_t), hipMemcpyHostToDevice, st));
      HIP_TRY(launch_gather_cols_colmajor(basis.p, n, ld, perm_d.p, nx, evecs_out, rowinv, st));
      HIP_TRY(hipStreamSynchronize(st));  // `outpos` is pageable host memory
    } else if (nx > 0) {
      std::vector<double> G((size_t)nx * nx, 0.0), hbuf((size_t)nx * kPP);
      const ProjectPlan plan = plan_project(n, nx, kMaxPartials);
      // columns [nx, nx+b) are zeroed so that a last chunk narrower than b is padded with zeros;
      // the products land in columns [nx+b, nx+2b)
      HIP_TRY(hipMemsetAsync(z.p, 0, (size_t)n * b * sizeof(double), st));
      HIP_TRY(launch_copy_cols(z.p, b, 0, basis.p, ld, nx, b, n, st));
      for (int c0 = 0; c0 < nx; c0 += b) {
        const int w = std::min(b, nx - c0);
        HIP_TRY(launch_pack_scaled(basis.p + c0, ld, zs(), n, b, z.p, st));
        spmm_from_z(basis.p + nx + b, ld);
        HIP_TRY(launch_project(basis.p, n, ld, 0, nx, nx + b, b, plan, part.p, st));
        HIP_TRY(launch_reduce_partials(part.p, plan.npart, nx, b, h1.p, nullptr, 0, nullptr, 0, st));
        HIP_TRY(hipMemcpyAsync(hbuf.data(), h1.p, (size_t)nx * kPP * sizeof(double), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        for (int r = 0; r < nx; ++r)
          for (int t = 0; t < w; ++t) G[(size_t)r * nx + c0 + t] = hbuf[(size_t)r * kPP + t];
        stats.spmv_cols += w;
      }
      const double te0 = now_s();
      SelectedEig rr;
      if (rr.factor(G.data(), nx) != 0) SC_THROW(SC_EHIP);
      const std::vector<double>& th = rr.values();
      std::vector<int> idx(nfound);
      for (int t = 0; t < nfound; ++t) idx[t] = nx - 1 - t;
      std::vector<double> yk((size_t)nx * nfound);  // column t = Ritz vector of the t-th largest theta
      rr.vectors(idx.data(), nfound, yk.data());
      stats.t_host_eig += now_s() - te0;
      stats.host_eigs += 1;
      for (int t = 0; t < nfound; ++t) evals_host[t] = 1.0 - th[nx - 1 - t];
      if ((size_t)nx * nfound > yd_cap) SC_THROW(SC_EDOMAIN);
      HIP_TRY(hipMemcpyAsync(yd.p, yk.data(), yk.size() * sizeof(double), hipMemcpyHostToDevice, st));
      HIP_TRY(launch_row_gemm(basis.p, n, ld, 0, nx, yd.p, nfound, nfound, 2, 0, evecs_out, n, rowmap, st));
      HIP_TRY(hipStreamSynchronize(st));
    }
    // the paper's Step 3 asks for the eigenvectors of L_n = D^-1 L: u = D^-1/2 v
    if ((flags & SC_FLAG_RANDOM_WALK_VECTORS) && nfound > 0)
      HIP_TRY(launch_scale_rows_colmajor(evecs_out, n, nfound, s.p, rowinv, st));
    // the embedding handed to k-means (Section II Step 4) with every point on the unit sphere
    if ((flags & SC_FLAG_ROW_NORMALIZE) && nfound > 0) HIP_TRY(launch_normalize_rows_colmajor(evecs_out, n, nfound, st));
    HIP_TRY(hipMemcpyAsync(evals_out, evals_host.data(), (size_t)k_out * sizeof(double), hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (debug_on()) std::fprintf(stderr, "[sceig] t=%.4fs outputs written\n", now_s() - t_begin);

    // the k_out returned pairs are the leading ones of the locked set: count and bound those
    int nconv = 0;
    double maxr = 0.0;
    {
      std::vector<int> byth(rho_locked.size());
      std::iota(byth.begin(), byth.end(), 0);
      std::stable_sort(byth.begin(), byth.end(), [&](int x, int y) { return theta_locked[x] > theta_locked[y]; });
      for (size_t t = 0; t < byth.size() && (int)t < k_out; ++t) {
        if (rho_locked[byth[t]] <= tol) ++nconv;
        maxr = std::max(maxr, rho_locked[byth[t]]);
      }
    }
    stats.nconv = std::min(nconv, k_out);
    stats.max_residual_est = maxr;
    stats.block = b;
    stats.m = m;
    timer.collect(&stats);
    stats.t_total = now_s() - t_begin;
    if (nfound < k_out) not_converged = true;
    return not_converged ? SC_NOT_CONVERGED : SC_OK;
  }
};

int guarded(int (*fn)(void*), void* ctx) {
  try {
    return fn(ctx);
  } catch (const ScError& e) {
    return e.code;
  } catch (const std::bad_alloc&) {
    return SC_ENOMEM;
  } catch (...) {
    return SC_EHIP;
  }
}

bool supported_block(int b) { return b == 1 || b == 2 || b == 4 || b == 8 || b == 16 || b == 32; }

}  // namespace
}  // namespace sceig

using namespace sceig;

// Basis budget m and block size b of a solve: the caller's values, or the defaults.
int resolve_basis(int64_t n, int32_t k, const sc_options& o, int64_t* m_out, int* b_out) {
  int64_t m = o.m;
  if (m == 0) m = std::min<int64_t>(n, std::max<int64_t>(2 * (int64_t)k, (int64_t)k + 56));
  if (m > n || m < (int64_t)k + 3) return SC_EDOMAIN;
  int b = o.block;
  if (b == 0) {
    // Larger blocks amortise the passes over the basis (their cost grows with n), smaller blocks keep the
    // projected problems and the number of block steps per converged vector small.
    int target = n >= 20000 ? 16 : 8;
    if (n >= 300000 && k >= 1000) target = 32;
    b = std::min(target, pow2_floor((int)std::max<int64_t>(1, (m - k) / 3)));
    int kb = 1;
    while (kb < k) kb *= 2;
    b = std::min(b, kb);
  }
  if (!supported_block(b) || (int64_t)k + 3 * (int64_t)b > m) return SC_EDOMAIN;
  *m_out = m;
  *b_out = b;
  return SC_OK;
}

// ---- k-means on the embedding (Section II Step 4, Section IV-C, Algorithms 4 and 5) ------------------------------
namespace {

// Counter-based uniform numbers in [0, 1) for the seeding draws: top 53 bits of mix(mix(seed) + index).
uint64_t km_mix64(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
double km_uniform01(uint64_t seed, uint64_t index) {
  return (double)(km_mix64(km_mix64(seed) + index) >> 11) * (1.0 / 9007199254740992.0);
}

struct KMeans {
  const double* points;
  int64_t ld;
  int colmajor;
  int64_t n;
  int d, k;
  hipStream_t st;
  int64_t ldx = 0;
  DevBuf<double> x;

  void stage() {  // row-major, zero padded, 32-byte aligned rows: the left operand of the distance product
    ldx = ((int64_t)d + 3) / 4 * 4;
    x.alloc((size_t)n * ldx);
    HIP_TRY(launch_points_to_rowmajor(points, ld, colmajor, n, d, x.p, ldx, st));
  }

  // Algorithm 5: chosen (device int32[k]) and the chosen points as centres (device k x ldx)
  void seed(uint64_t seed_value, int32_t* chosen, double* c) {
    std::vector<double> u((size_t)k);
    for (int i = 0; i < k; ++i) u[i] = km_uniform01(seed_value, (uint64_t)i);
    const size_t wb = kmeans_seed_workspace(n);
    DevBuf<char> work;
    work.alloc(wb);
    HIP_TRY(launch_kmeanspp(x.p, ldx, d, n, k, u.data(), work.p, wb, chosen, st));
    HIP_TRY(launch_gather_rows(x.p, ldx, chosen, k, c, st));
    HIP_TRY(hipStreamSynchronize(st));  // u and work are released on return
  }

  // Algorithm 4 step 3 from the centres in c (device k x ldx, updated in place)
  int lloyd(double* c, int max_iter, int32_t* labels, sc_kmeans_stats* stats) {
    const int64_t ldc = ((int64_t)k + 15) / 16 * 16;
    int64_t chunk = ((int64_t)1 << 27) / ldc / 128 * 128;  // distance block of at most 1 GiB
    if (chunk < 128) chunk = 128;
    if (chunk > n) chunk = n;
    DevBuf<double> ct, cnorm, sblock, part;
    DevBuf<int32_t> start;
    DevBuf<int> changes;
    DevBuf<char> work;
    PinnedBuf<int> hchanges;
    ct.alloc((size_t)ldx * ldc);
    cnorm.alloc((size_t)k);
    sblock.alloc((size_t)chunk * ldc);
    start.alloc((size_t)k + 1);
    changes.alloc(1);
    hchanges.alloc(1);
    const size_t wb = kmeans_update_workspace(n);
    work.alloc(wb);
    HIP_TRY(launch_fill_int32(labels, n, -1, 0, st));
    int iters = 0, converged = 0, last_changes = 0;
    const bool timing = stats && stats->timing;
    struct EventPair {
      hipEvent_t a, b;
    };
    struct EventList {  // destroys what it still holds, also when an error unwinds the call
      std::vector<EventPair> v;
      ~EventList() {
        for (EventPair& e : v) {
          if (e.a) (void)hipEventDestroy(e.a);
          if (e.b) (void)hipEventDestroy(e.b);
        }
      }
    } events;
    double dist_bytes = 0.0, dist_flops = 0.0;
    for (int it = 0; it < max_iter; ++it) {
      HIP_TRY(launch_fill_int32(changes.p, 1, 0, 0, st));
      HIP_TRY(launch_centroid_operand(c, ldx, k, d, (int)ldx, ct.p, ldc, cnorm.p, st));
      for (int64_t r0 = 0; r0 < n; r0 += chunk) {
        const int64_t rows = std::min<int64_t>(chunk, n - r0);
        if (timing) {
          events.v.push_back(EventPair{nullptr, nullptr});
          HIP_TRY(hipEventCreate(&events.v.back().a));
          HIP_TRY(hipEventCreate(&events.v.back().b));
          HIP_TRY(hipEventRecord(events.v.back().a, st));
        }
        HIP_TRY(launch_row_gemm(x.p + r0 * ldx, rows, ldx, 0, d, ct.p, (int)ldc, k, 1, 0, sblock.p, ldc, nullptr, st));
        if (timing) HIP_TRY(hipEventRecord(events.v.back().b, st));
        dist_bytes += 8.0 * ((double)rows * d + (double)rows * k + (double)k * d);
        dist_flops += 2.0 * (double)rows * k * d;
        HIP_TRY(launch_argmin(sblock.p, ldc, rows, k, cnorm.p, labels + r0, changes.p, st));
      }
      HIP_TRY(hipMemcpyAsync(hchanges.p, changes.p, sizeof(int), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      ++iters;
      last_changes = *hchanges.p;
      if (last_changes == 0) {
        converged = 1;
        break;
      }
      HIP_TRY(launch_centroid_update(x.p, ldx, d, n, labels, k, work.p, wb, start.p, c, st));
    }
    if (stats) {
      // objective of the final labelling against the centres it was computed from (after a converged run these are
      // also the means of their clusters)
      const int np = kmeans_objective_parts();
      part.alloc((size_t)np);
      std::vector<double> hp((size_t)np);
      if (converged || max_iter == 0 || iters == 0) {
        HIP_TRY(launch_objective(x.p, ldx, d, n, labels, c, part.p, st));
        HIP_TRY(hipMemcpyAsync(hp.data(), part.p, sizeof(double) * np, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        double tot = 0.0;
        for (int p = 0; p < np; ++p) tot += hp[p];
        stats->objective = tot;
      } else {
        stats->objective = -1.0;  // the centres moved after the last labelling
      }
      stats->iterations = iters;
      stats->converged = converged;
      stats->last_changes = last_changes;
      stats->distance_launches = (int64_t)(timing ? events.v.size() : 0);
      stats->distance_bytes = dist_bytes;
      stats->distance_flops = dist_flops;
      double td = 0.0;
      for (EventPair& ev : events.v) {  // every launch has completed: the stream was synchronized above
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ev.a, ev.b) == hipSuccess) td += ms * 1e-3;
      }
      stats->t_distance = td;
    }
    return converged ? SC_OK : SC_NOT_CONVERGED;
  }
};

struct KMeansCall {
  KMeans km;
  uint64_t seed;
  int max_iter;
  int mode;  // 0 = seeding only, 1 = Lloyd from given centres, 2 = both
  int32_t* chosen_out;
  int32_t* labels_out;
  double* centroids;  // k x d row-major, caller's
  sc_kmeans_stats* stats;
};

int run_kmeans(void* p) {
  KMeansCall* c = static_cast<KMeansCall*>(p);
  KMeans& km = c->km;
  const auto t0 = std::chrono::steady_clock::now();
  km.stage();
  DevBuf<double> cen;
  DevBuf<int32_t> chosen;
  cen.alloc((size_t)km.k * km.ldx);
  double t_seed = 0.0;
  if (c->mode != 1) {
    int32_t* ch = c->chosen_out;
    if (!ch) {
      chosen.alloc((size_t)km.k);
      ch = chosen.p;
    }
    km.seed(c->seed, ch, cen.p);
    t_seed = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  } else {
    HIP_TRY(launch_points_to_rowmajor(c->centroids, km.d, 0, km.k, km.d, cen.p, km.ldx, km.st));
  }
  int rc = SC_OK;
  if (c->mode != 0) rc = km.lloyd(cen.p, c->max_iter, c->labels_out, c->stats);
  HIP_TRY(launch_copy_rows(cen.p, km.ldx, c->centroids, km.d, km.k, km.d, km.st));
  HIP_TRY(hipStreamSynchronize(km.st));
  if (c->stats) {
    c->stats->t_seed = t_seed;
    c->stats->t_total = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  }
  return rc;
}

int kmeans_args_ok(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k) {
  if (!points || n < 0 || ld < 0) return SC_EINVAL;
  if (n < 1 || n > (int64_t)0x7fffffff / 16 || d < 1 || k < 1 || (int64_t)k > n) return SC_EDOMAIN;
  if (ld < (colmajor ? n : (int64_t)d)) return SC_EDOMAIN;
  return SC_OK;
}

}  // namespace

namespace {

// Block QR on caller-visible scratch: part (kMaxPartials * b * kPP doubles), gpart (kGramPartials * kPP * kPP) and
// small (5 * kPP * kPP).  Every entry of the scratch is written by a kernel before a kernel reads it, so its contents
// on entry do not matter.
void run_block_qr(double* basis, int64_t n, int64_t ld, int j, int b, double* r_out, double* g_out, double* part,
                  double* gpart, double* small, hipStream_t st) {
  double* rinv = small;
  double* r1 = small + kPP * kPP;
  double* rr = small + 2 * kPP * kPP;
  double* gg = small + 3 * kPP * kPP;
  double* gram = small + 4 * kPP * kPP;
  enqueue_block_qr(basis, n, ld, j, b, part, gpart, 0, gram, rinv, r1, rr, gg, nullptr, nullptr, st, nullptr);
  const size_t w = (size_t)b * sizeof(double);
  if (r_out)
    HIP_TRY(hipMemcpy2DAsync(r_out, w, rr, (size_t)kPP * sizeof(double), w, (size_t)b, hipMemcpyDeviceToDevice, st));
  if (g_out)
    HIP_TRY(hipMemcpy2DAsync(g_out, w, gg, (size_t)kPP * sizeof(double), w, (size_t)b, hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));
}

struct BlockQrCall {
  double* basis;
  int64_t n, ld;
  int j, b;
  double *r, *g;
  hipStream_t st;
};

// Scratch of sc_block_qr_noalloc: device memory that lives in the library's code object, one copy per GPU, from the
// moment the library is loaded on it until the process ends.  Sized for the largest block (32 columns): the partial
// Gram blocks of the projection (512) and of the fused scaling pass (1024) and five small matrices.
constexpr size_t kQrPartDoubles = (size_t)kMaxPartials * kMaxBlock * kPP;
constexpr size_t kQrGpartDoubles = (size_t)kGramPartials * kPP * kPP;
constexpr size_t kQrSmallDoubles = (size_t)5 * kPP * kPP;
constexpr size_t kQrScratchDoubles = kQrPartDoubles + kQrGpartDoubles + kQrSmallDoubles;

}  // namespace

static __device__ __align__(256) double scratch[kQrScratchDoubles];

namespace {

// The array's name is only a handle in host code; its address on a device comes from the runtime, once per device.
constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
double* scratch_ptr[kMaxDevices] = {};

double* scratch_on_current_device() {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) SC_THROW(SC_EDOMAIN);
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) SC_THROW(SC_EHIP);
    scratch_ptr[dev] = static_cast<double*>(p);
  }
  return scratch_ptr[dev];
}

}  // namespace

extern "C" {

int sc_version(void) { return 100; }

int64_t sc_counter(int32_t which) {
  switch (which) {
    case SC_COUNTER_RESIDENT_FILTERS: return resident_launches.load(std::memory_order_relaxed);
    default: return -1;
  }
}

int sc_probe_fp64_matrix_rate(int32_t shape, int32_t workgroups, int32_t iterations, double* tflops_out, void* stream) {
  if (!tflops_out) return SC_EINVAL;
  if (shape != 4 && shape != 16) return SC_EDOMAIN;
  if (workgroups < 1 || workgroups > (1 << 20) || iterations < 1 || iterations > (1 << 24)) return SC_EDOMAIN;
  struct Ctx {
    int shape, wgs, iters;
    double* out;
    hipStream_t st;
  } ctx{shape, workgroups, iterations, tflops_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        DevBuf<double> sink;
        sink.alloc((size_t)c->wgs * 256);
        hipEvent_t e0 = nullptr, e1 = nullptr;
        HIP_TRY(launch_mfma_rate(sink.p, c->shape, c->wgs, 64, c->st));  // warm-up: code object loaded, clocks up
        HIP_TRY(hipEventCreate(&e0));
        hipError_t err = hipEventCreate(&e1);
        if (err == hipSuccess) err = hipEventRecord(e0, c->st);
        if (err == hipSuccess) err = launch_mfma_rate(sink.p, c->shape, c->wgs, c->iters, c->st);
        if (err == hipSuccess) err = hipEventRecord(e1, c->st);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        (void)hipStreamSynchronize(c->st);  // the sink goes back to the cache only after the kernel has finished
        (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        HIP_TRY(err);
        const double flops = (double)c->wgs * 4.0 * (double)c->iters * 8.0 * (c->shape == 16 ? 2048.0 : 512.0);
        *c->out = ms > 0.0f ? flops / ((double)ms * 1e-3) / 1e12 : 0.0;
        return SC_OK;
      },
      &ctx);
}

int sc_release_cache(void) {
  device_cache().clear();
  pinned_cache().clear();
  return SC_OK;
}

const char* sc_strerror(int code) {
  switch (code) {
    case SC_OK: return "ok";
    case SC_NOT_CONVERGED: return "not converged within maxiter restart cycles";
    case SC_EINVAL: return "invalid argument (null pointer or negative size)";
    case SC_EDOMAIN: return "argument out of domain (k, m, block or tol)";
    case SC_ECSR: return "malformed CSR";
    case SC_EZERODEG: return "a node has a non-positive or non-finite degree";
    case SC_ENOMEM: return "out of memory";
    case SC_EHIP: return "HIP runtime failure";
    case SC_EINTERNAL: return "an internal iteration limit was exceeded";
    default: return "unknown code";
  }
}

namespace {

int eigsh_entry(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n, int32_t k, double tol,
                int32_t maxiter, double* evals_out, double* evecs_out, void* stream, const sc_options* opt, sc_stats* stats,
                void* workspace, size_t workspace_bytes, bool use_workspace) {
  if (!csr_rowptr || !csr_col || !csr_val || !evals_out || !evecs_out || n < 0) return SC_EINVAL;
  if (use_workspace && !workspace) return SC_EINVAL;
  sc_options o{};
  if (opt) o = *opt;
  if (k < 1 || o.guard < 0 || (int64_t)k + o.guard >= n || !(tol >= 0.0) || maxiter < 1) return SC_EDOMAIN;
  if (n > (int64_t)0x7fffffff) return SC_EDOMAIN;
  const int kk = k + o.guard;
  int64_t m = 0;
  int b = 0;
  const int rc0 = resolve_basis(n, kk, o, &m, &b);
  if (rc0 != SC_OK) return rc0;
  Arena arena(workspace, workspace_bytes);  // outlives the solver, whose blocks point into it
  Solver sv;
  sv.rowptr = csr_rowptr;
  sv.col = csr_col;
  sv.val = csr_val;
  sv.n = n;
  sv.nnz = 0;
  sv.k = kk;
  sv.k_out = k;
  sv.tol = tol;
  sv.maxiter = maxiter;
  sv.flags = o.flags;
  sv.timer.mask = o.timing_mask;
  sv.seed = o.seed;
  sv.v0 = o.v0;
  sv.check_every = o.check_every > 0 ? o.check_every : 2;
  sv.st = reinterpret_cast<hipStream_t>(stream);
  sv.m = (int)m;
  sv.b = b;
  sv.ws_limit = use_workspace ? std::max<size_t>(workspace_bytes, 1) : 0;
  struct Ctx {
    Solver* sv;
    double* ev;
    double* evec;
    Arena* arena;
  } ctx{&sv, evals_out, evecs_out, use_workspace ? &arena : nullptr};
  const int rc = guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        struct Install {  // the workspace serves every device block of this call, on this thread only
          explicit Install(Arena* a) { tl_arena = a; }
          ~Install() { tl_arena = nullptr; }
        } install(c->arena);
        return c->sv->run(c->ev, c->evec);
      },
      &ctx);
  if (stats) *stats = sv.stats;
  if (rc < 0) (void)hipStreamSynchronize(sv.st);
  if (use_workspace && debug_on())
    std::fprintf(stderr, "[sceig] workspace: %zu bytes given, high-water mark %zu\n", workspace_bytes, arena.peak());
  return rc;
}

}  // namespace

int sc_laplacian_eigsh(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n, int32_t k,
                       double tol, int32_t maxiter, double* evals_out, double* evecs_out, void* stream,
                       const sc_options* opt, sc_stats* stats) {
  return eigsh_entry(csr_rowptr, csr_col, csr_val, n, k, tol, maxiter, evals_out, evecs_out, stream, opt, stats, nullptr, 0,
                     false);
}

int sc_laplacian_eigsh_ws(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n, int32_t k,
                          double tol, int32_t maxiter, double* evals_out, double* evecs_out, void* stream,
                          const sc_options* opt, sc_stats* stats, void* workspace, size_t workspace_bytes) {
  return eigsh_entry(csr_rowptr, csr_col, csr_val, n, k, tol, maxiter, evals_out, evecs_out, stream, opt, stats, workspace,
                     workspace_bytes, true);
}

int sc_workspace_bytes(int64_t n, int64_t nnz, int32_t k, const sc_options* opt, size_t* bytes_out) {
  if (!bytes_out || n < 0 || nnz < 0) return SC_EINVAL;
  sc_options o{};
  if (opt) o = *opt;
  if (k < 1 || o.guard < 0 || (int64_t)k + o.guard >= n || n > (int64_t)0x7fffffff) return SC_EDOMAIN;
  k += o.guard;  // the iteration works for k + guard pairs
  int64_t m = 0;
  int b = 0;
  const int rc = resolve_basis(n, k, o, &m, &b);
  if (rc != SC_OK) return rc;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t N = (size_t)n, Z = (size_t)nnz;
  const size_t ld = ((size_t)m + b + 15) / 16 * 16;
  const size_t jmax = (size_t)m + b;
  const size_t rot_cols = (size_t)std::min<int64_t>(m, std::max<int64_t>(m / 2 + b, 2 * (int64_t)b));
  size_t total = 0;
  if (!(o.flags & SC_FLAG_NO_REORDER)) {
    // the renumbered operator copy, the two row maps, and the sort's scratch (released before the basis is allocated,
    // but held while the copy is built)
    total += up((N + 1) * 8) + up(Z * 4) + up(Z * 8) + 2 * up(N * 4);
    total += up(order_by_component_workspace(n)) + 2 * up(N * 4);
  }
  total += up(N * 8);                       // scaling vector
  if (b >= 8) total += up(Z * 8) + up(N * 4) + up(long_row_list_workspace(n)) + 256;  // scaled values, long-row list
  if (b >= 8 && !(o.flags & SC_FLAG_NO_START_FILTER))  // diagonal-block search and the work items of the resident filter
    total += up(diagonal_blocks_workspace(n)) + up(N * 4) + 256 + up(N * 8) + up(N * 18) +
             up(Z * 15 + N * 2) + up(Z * 3 + N / 4) + 5 * up(N / 8 + 64) + up(sliced_scan_workspace((int)std::min<int64_t>(n, INT32_MAX)));  // + sliced copy (at most 1.5 x the entries plus look-ahead rounds) and its slice tables
  total += up(N * ld * 8) + up(N * (size_t)b * 8) + up(N * rot_cols * 8);  // basis, packed block, rotation workspace
  total += up((size_t)kMaxPartials * jmax * kPP * 8) + up((size_t)kGramPartials * kPP * kPP * 8) + 2 * up(jmax * kPP * 8);
  total += up((size_t)(m / b + 4) * kSlotDoubles * 8) + up(jmax * std::max<size_t>(rot_cols, (size_t)k) * 8);
  if (o.flags & SC_FLAG_COMPONENT_NULLSPACE) total += up(N * 8) + up(N * 4) + up(N * 8);
  total += up((size_t)3 * kPP * kPP * 8) + up((size_t)k * 4);  // small matrices, the output permutation
  total += 16 * 256;                        // flags and counters, alignment of the caller's workspace
  *bytes_out = total;
  return SC_OK;
}

int sc_degree_scaling(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                      double* d_out, double* s_out, void* stream) {
  (void)csr_col;
  if (!csr_rowptr || !csr_val || !s_out || n < 0) return SC_EINVAL;
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const double* v;
    int64_t n;
    double *d, *s;
    hipStream_t st;
  } ctx{csr_rowptr, csr_val, n, d_out, s_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        DevBuf<int> flag;
        flag.alloc(1);
        HIP_TRY(hipMemsetAsync(flag.p, 0, sizeof(int), c->st));
        HIP_TRY(launch_degree_scaling(c->rp, c->v, c->n, c->d, c->s, flag.p, c->st));
        int h = 0;
        HIP_TRY(hipMemcpyAsync(&h, flag.p, sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return (h & 4) ? SC_EZERODEG : SC_OK;
      },
      &ctx);
}

int sc_validate_csr(const int64_t* csr_rowptr, const int32_t* csr_col, int64_t n, void* stream) {
  if (!csr_rowptr || !csr_col || n < 0) return SC_EINVAL;
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    int64_t n;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, n, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        int64_t nnz = 0;
        HIP_TRY(hipMemcpyAsync(&nnz, c->rp + c->n, sizeof(int64_t), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        if (nnz < 0) return SC_ECSR;
        DevBuf<int> flag;
        flag.alloc(1);
        HIP_TRY(hipMemsetAsync(flag.p, 0, sizeof(int), c->st));
        HIP_TRY(launch_validate_csr(c->rp, c->c, c->n, nnz, flag.p, c->st));
        int h = 0;
        HIP_TRY(hipMemcpyAsync(&h, flag.p, sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return (h & 3) ? SC_ECSR : SC_OK;
      },
      &ctx);
}

int sc_reorder_csr(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                   int64_t* rowptr_out, int32_t* col_out, double* val_out, int32_t* old_of_new_out, int32_t* ncomp_out,
                   void* stream) {
  if (!csr_rowptr || !csr_col || !csr_val || !rowptr_out || !col_out || !val_out || !old_of_new_out || n < 0)
    return SC_EINVAL;
  if (n > (int64_t)0x7fffffff) return SC_EDOMAIN;
  if (ncomp_out) *ncomp_out = 0;
  if (n == 0) return SC_OK;
  const int rc = sc_validate_csr(csr_rowptr, csr_col, n, stream);
  if (rc != SC_OK) return rc;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    const double* v;
    int64_t n;
    int64_t* rpo;
    int32_t* co;
    double* vo;
    int32_t* oon;
    int32_t* nc;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, csr_val, n, rowptr_out, col_out, val_out, old_of_new_out, ncomp_out,
        reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        int64_t nnz = 0;
        HIP_TRY(hipMemcpyAsync(&nnz, c->rp + c->n, sizeof(int64_t), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        const int ncomp = reorder_csr(c->rp, c->c, c->v, c->n, nnz, c->rpo, c->co, c->vo, c->oon, nullptr, nullptr, 0, c->st);
        if (c->nc) *c->nc = ncomp;
        return SC_OK;
      },
      &ctx);
}

int sc_spmm_normalized(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                       int64_t n, const double* x, int64_t ldx, double* y, int64_t ldy, int32_t ncols, double* work,
                       void* stream) {
  if (!csr_rowptr || !csr_col || !csr_val || !x || !y || n < 0) return SC_EINVAL;
  if (!supported_block(ncols) || ldx < ncols || ldy < ncols) return SC_EDOMAIN;
  if (reinterpret_cast<uintptr_t>(work) % 16 != 0) return SC_EINVAL;  // the product gathers 16-byte pieces of it
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    const double* v;
    const double* s;
    int64_t n;
    const double* x;
    int64_t ldx;
    double* y;
    int64_t ldy;
    int b;
    double* work;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, csr_val, s, n, x, ldx, y, ldy, ncols, work, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        DevBuf<double> own;
        // s == null: the values are the scaled operator and the operand needs no scaling; if it is already packed
        // (and 16-byte aligned, which the wide products' gathers need) it is gathered from where it is
        const bool in_place = !c->s && c->ldx == c->b && reinterpret_cast<uintptr_t>(c->x) % 16 == 0;
        double* z = c->work;
        if (!z && !in_place) {
          own.alloc((size_t)c->n * c->b);
          z = own.p;
        }
        // the entry count only steers the kernel choice; it is remembered for the last graph seen so that
        // repeated products with one matrix do not pay a device-to-host round trip each
        static thread_local const int64_t* last_rp = nullptr;
        static thread_local const int32_t* last_col = nullptr;
        static thread_local const double* last_val = nullptr;
        static thread_local int64_t last_n = -1, last_nnz = 0;
        if (last_rp != c->rp || last_col != c->c || last_val != c->v || last_n != c->n) {
          int64_t nnz = 0;
          HIP_TRY(hipMemcpyAsync(&nnz, c->rp + c->n, sizeof(int64_t), hipMemcpyDeviceToHost, c->st));
          HIP_TRY(hipStreamSynchronize(c->st));
          last_rp = c->rp;
          last_col = c->c;
          last_val = c->v;
          last_n = c->n;
          last_nnz = nnz;
        }
        if (!in_place) HIP_TRY(launch_pack_scaled(c->x, c->ldx, c->s, c->n, c->b, z, c->st));
        HIP_TRY(launch_spmm(c->rp, c->c, c->v, c->s, c->n, in_place ? c->x : z, c->b, c->y, c->ldy,
                            (double)last_nnz / (double)c->n, c->st));
        if (own.p) HIP_TRY(hipStreamSynchronize(c->st));  // the internal scratch is freed on return
        return SC_OK;
      },
      &ctx);
}

int sc_spmv_normalized_chain(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                             int64_t n, int64_t nnz, const double* z_in, double* y, double* z_out, void* stream) {
  if (!csr_rowptr || !csr_col || !csr_val || !s || !z_in || !y || !z_out || n < 0 || nnz < 0) return SC_EINVAL;
  if (z_out == z_in || y == z_in) return SC_EINVAL;  // rows gather the operand of other rows
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    const double *v, *s;
    int64_t n, nnz;
    const double* z;
    double *y, *zo;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, csr_val, s, n, nnz, z_in, y, z_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        HIP_TRY(launch_spmv_chain(c->rp, c->c, c->v, c->s, c->n, c->z, c->y, c->zo, (double)c->nnz / (double)c->n, c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_scale_operator(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, const double* s,
                      int64_t n, double* val_out, void* stream) {
  if (!csr_rowptr || !csr_col || !csr_val || !s || !val_out || n < 0) return SC_EINVAL;
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    const double *v, *s;
    int64_t n;
    double* out;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, csr_val, s, n, val_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        HIP_TRY(launch_scale_values(c->rp, c->c, c->v, c->s, c->out, c->n, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_cgs2(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* h_out, double* gram_out, void* stream) {
  if (!basis || n < 0) return SC_EINVAL;
  if (b < 1 || b > kMaxBlock || j < 0 || ld < (int64_t)j + b) return SC_EDOMAIN;
  if (n == 0 || j == 0) return SC_OK;
  struct Ctx {
    double* basis;
    int64_t n, ld;
    int j, b;
    double *h, *g;
    hipStream_t st;
  } ctx{basis, n, ld, j, b, h_out, gram_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        DevBuf<double> part, h1, hsum, gpart, gram;
        part.alloc((size_t)kMaxPartials * c->j * kPP);
        h1.alloc((size_t)c->j * kPP);
        hsum.alloc((size_t)c->j * kPP);
        gpart.alloc((size_t)kGramPartials * kPP * kPP);
        gram.alloc((size_t)kPP * kPP);
        const int ngram =
            enqueue_cgs2(c->basis, c->n, c->ld, c->j, c->j, c->b, 0, part.p, h1.p, hsum.p, nullptr, 0, gpart.p, c->st, nullptr);
        const size_t w = (size_t)c->b * sizeof(double);
        if (c->h)
          HIP_TRY(hipMemcpy2DAsync(c->h, w, hsum.p, (size_t)kPP * sizeof(double), w, (size_t)c->j,
                                   hipMemcpyDeviceToDevice, c->st));
        if (c->g) {
          HIP_TRY(launch_reduce_partials(gpart.p, ngram, c->b, c->b, gram.p, nullptr, 0, nullptr, 0, c->st));
          HIP_TRY(hipMemcpy2DAsync(c->g, w, gram.p, (size_t)kPP * sizeof(double), w, (size_t)c->b,
                                   hipMemcpyDeviceToDevice, c->st));
        }
        HIP_TRY(hipStreamSynchronize(c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_block_qr(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* r_out, double* g_out,
                void* stream) {
  if (!basis || n < 0) return SC_EINVAL;
  if (!supported_block(b) || j < 0 || ld < (int64_t)j + b) return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  BlockQrCall ctx{basis, n, ld, j, b, r_out, g_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        BlockQrCall* c = static_cast<BlockQrCall*>(p);
        DevBuf<double> part, small, gpart;
        part.alloc((size_t)kMaxPartials * c->b * kPP);
        gpart.alloc(kQrGpartDoubles);
        small.alloc(kQrSmallDoubles);
        run_block_qr(c->basis, c->n, c->ld, c->j, c->b, c->r, c->g, part.p, gpart.p, small.p, c->st);
        return SC_OK;
      },
      &ctx);
}

int sc_block_qr_noalloc(double* basis, int64_t n, int64_t ld, int32_t j, int32_t b, double* r_out, double* g_out,
                        void* stream) {
  if (!basis || n < 0) return SC_EINVAL;
  // the scratch holds the partial blocks of a block of at most kMaxBlock columns, whatever n is
  if (!supported_block(b) || b > kMaxBlock || j < 0 || ld < (int64_t)j + b || n > (int64_t)0x7fffffff) return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  BlockQrCall ctx{basis, n, ld, j, b, r_out, g_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        BlockQrCall* c = static_cast<BlockQrCall*>(p);
        double* sp = scratch_on_current_device();
        run_block_qr(c->basis, c->n, c->ld, c->j, c->b, c->r, c->g, sp, sp + kQrPartDoubles,
                     sp + kQrPartDoubles + kQrGpartDoubles, c->st);
        return SC_OK;
      },
      &ctx);
}

int sc_rotate(const double* basis, int64_t n, int64_t ld, int32_t j0, int32_t ja, const double* y, int32_t l,
              double* out, int64_t ldo, int32_t out_colmajor, void* stream) {
  if (!basis || !y || !out || n < 0) return SC_EINVAL;
  if (j0 < 0 || ja < 1 || l < 1 || ld < (int64_t)j0 + ja) return SC_EDOMAIN;
  if (out_colmajor ? (ldo < n) : (ldo < l)) return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  struct Ctx {
    const double* basis;
    int64_t n, ld;
    int j0, ja;
    const double* y;
    int l;
    double* out;
    int64_t ldo;
    int cm;
    hipStream_t st;
  } ctx{basis, n, ld, j0, ja, y, l, out, ldo, out_colmajor, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        HIP_TRY(launch_row_gemm(const_cast<double*>(c->basis), c->n, c->ld, c->j0, c->ja, c->y, c->l, c->l,
                                c->cm ? 2 : 1, 0, c->out, c->ldo, nullptr, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_chebyshev_filter(const int64_t* csr_rowptr, const int32_t* csr_col, const double* csr_val, int64_t n,
                        const double* x, int64_t ldx, int32_t ncols, double a, int32_t degree, double* y, int64_t ldy,
                        void* stream) {
  if (!csr_rowptr || !csr_col || !csr_val || !x || !y || n < 0) return SC_EINVAL;
  if (!supported_block(ncols) || ldx < ncols || ldy < ncols || degree < 1 || !(a > -1.0) || !(a < 1.0))
    return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  struct Ctx {
    const int64_t* rp;
    const int32_t* c;
    const double* v;
    int64_t n;
    const double* x;
    int64_t ldx;
    int b;
    double a;
    int d;
    double* y;
    int64_t ldy;
    hipStream_t st;
  } ctx{csr_rowptr, csr_col, csr_val, n, x, ldx, ncols, a, degree, y, ldy, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        int64_t nnz = 0;
        HIP_TRY(hipMemcpyAsync(&nnz, c->rp + c->n, sizeof(int64_t), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        if (nnz < 0) SC_THROW(SC_ECSR);
        DevBuf<double> s, vals, z, b1, b2, b3;
        DevBuf<int> flag;
        flag.alloc(1);
        HIP_TRY(hipMemsetAsync(flag.p, 0, sizeof(int), c->st));
        s.alloc((size_t)c->n);
        HIP_TRY(launch_degree_scaling(c->rp, c->v, c->n, nullptr, s.p, flag.p, c->st));
        int hflag = 0;
        HIP_TRY(hipMemcpyAsync(&hflag, flag.p, sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        if (hflag & 4) SC_THROW(SC_EZERODEG);
        const size_t blk = (size_t)c->n * c->b;
        z.alloc(blk);
        b1.alloc(blk);
        b2.alloc(blk);
        const bool wide = c->b >= 8;
        if (wide) {
          vals.alloc((size_t)nnz);
          HIP_TRY(launch_scale_values(c->rp, c->c, c->v, s.p, vals.p, c->n, c->st));
          HIP_TRY(launch_pack_scaled(c->x, c->ldx, nullptr, c->n, c->b, z.p, c->st));
        } else {
          b3.alloc(blk);
          HIP_TRY(launch_pack_scaled(c->x, c->ldx, s.p, c->n, c->b, z.p, c->st));
          HIP_TRY(launch_pack_scaled(c->x, c->ldx, nullptr, c->n, c->b, b1.p, c->st));
        }
        DevBuf<int32_t> longrows, lcount;
        int nlong = 0;
        if (wide) {  // the rows the wide product hands to whole workgroups, as in the solver's setup
          const size_t lw = long_row_list_workspace(c->n);
          DevBuf<char> lwork;
          lwork.alloc(lw);
          lcount.alloc(1);
          longrows.alloc((size_t)c->n);
          HIP_TRY(long_row_list(c->rp, c->n, lwork.p, lw, longrows.p, lcount.p, c->st));
          int32_t hcount = 0;
          HIP_TRY(hipMemcpyAsync(&hcount, lcount.p, sizeof(int32_t), hipMemcpyDeviceToHost, c->st));
          HIP_TRY(hipStreamSynchronize(c->st));
          nlong = hcount;
        }
        ResidentPlan resident;  // used when the matrix as given is block diagonal with blocks that fit LDS
        if (wide) plan_resident(c->rp, c->c, vals.p, c->n, nnz, c->b, c->st, &resident);
        const double* res = enqueue_cheb_filter(c->rp, c->c, c->v, wide ? vals.p : nullptr, s.p, c->n, nnz, c->b, c->d,
                                                c->a, z.p, b1.p, b2.p, b3.p, (double)nnz / (double)c->n,
                                                wide ? longrows.p : nullptr, nlong, &resident, c->st, nullptr);
        HIP_TRY(launch_copy_cols(res, c->b, 0, c->y, c->ldy, 0, c->b, c->n, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_kmeanspp(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k, uint64_t seed,
                int32_t* chosen_out, double* centroids_out, void* stream) {
  if (!centroids_out) return SC_EINVAL;
  const int a = kmeans_args_ok(points, ld, colmajor, n, d, k);
  if (a != SC_OK) return a;
  KMeansCall call{{points, ld, colmajor, n, d, k, reinterpret_cast<hipStream_t>(stream)}, seed, 0, 0, chosen_out, nullptr,
                  centroids_out, nullptr};
  return guarded(run_kmeans, &call);
}

int sc_kmeans_lloyd(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k,
                    double* centroids, int32_t max_iter, int32_t* labels_out, sc_kmeans_stats* stats, void* stream) {
  if (!centroids || !labels_out) return SC_EINVAL;
  const int a = kmeans_args_ok(points, ld, colmajor, n, d, k);
  if (a != SC_OK) return a;
  if (max_iter < 1) return SC_EDOMAIN;
  if (stats) {
    const int32_t timing = stats->timing;
    *stats = sc_kmeans_stats{};
    stats->timing = timing;
  }
  KMeansCall call{{points, ld, colmajor, n, d, k, reinterpret_cast<hipStream_t>(stream)}, 0, max_iter, 1, nullptr,
                  labels_out, centroids, stats};
  return guarded(run_kmeans, &call);
}

int sc_kmeans(const double* points, int64_t ld, int32_t colmajor, int64_t n, int32_t d, int32_t k, uint64_t seed,
              int32_t max_iter, int32_t* labels_out, double* centroids_out, sc_kmeans_stats* stats, void* stream) {
  if (!centroids_out || !labels_out) return SC_EINVAL;
  const int a = kmeans_args_ok(points, ld, colmajor, n, d, k);
  if (a != SC_OK) return a;
  if (max_iter < 1) return SC_EDOMAIN;
  if (stats) {
    const int32_t timing = stats->timing;
    *stats = sc_kmeans_stats{};
    stats->timing = timing;
  }
  KMeansCall call{{points, ld, colmajor, n, d, k, reinterpret_cast<hipStream_t>(stream)}, seed, max_iter, 2, nullptr,
                  labels_out, centroids_out, stats};
  return guarded(run_kmeans, &call);
}

int sc_edge_similarity(const double* x, int64_t ldx, int64_t n, int32_t d, const int32_t* edge_u, const int32_t* edge_v,
                       int64_t nedges, int32_t measure, double sigma, double* val_out, void* stream) {
  if (!x || n < 0 || nedges < 0 || (nedges > 0 && (!edge_u || !edge_v || !val_out))) return SC_EINVAL;
  if (d < 1 || ldx < d || measure < 0 || measure > 2 || (measure == 2 && !(sigma > 0.0))) return SC_EDOMAIN;
  if (nedges == 0 || n == 0) return nedges == 0 ? SC_OK : SC_EDOMAIN;
  struct Ctx {
    const double* x;
    int64_t ldx, n;
    int d;
    const int32_t *u, *v;
    int64_t ne;
    int measure;
    double sigma;
    double* val;
    hipStream_t st;
  } ctx{x, ldx, n, d, edge_u, edge_v, nedges, measure, sigma, val_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        DevBuf<double> mean, norm;
        DevBuf<int> bad;
        PinnedBuf<int> hbad;
        bad.alloc(1);
        hbad.alloc(1);
        HIP_TRY(launch_fill_int32(bad.p, 1, 0, 0, c->st));
        if (c->measure != 2) {
          mean.alloc((size_t)c->n);
          norm.alloc((size_t)c->n);
          HIP_TRY(launch_row_stats(c->x, c->ldx, c->n, c->d, c->measure == 0 ? 1 : 0, mean.p, norm.p, c->st));
        }
        HIP_TRY(launch_edge_similarity(c->x, c->ldx, c->d, c->u, c->v, c->ne, c->measure, c->sigma, mean.p, norm.p,
                                       c->n, bad.p, c->val, c->st));
        HIP_TRY(hipMemcpyAsync(hbad.p, bad.p, sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return *hbad.p ? SC_ECSR : SC_OK;
      },
      &ctx);
}

int sc_coo_to_csr(const int32_t* row, const int32_t* col, const double* val, int64_t nnz_in, int64_t n,
                  int32_t symmetrize, int64_t* rowptr_out, int32_t* col_out, double* val_out, int64_t* nnz_out,
                  void* stream) {
  if (!rowptr_out || n < 0 || nnz_in < 0 || (nnz_in > 0 && (!row || !col || !val || !col_out || !val_out)))
    return SC_EINVAL;
  if (n > (int64_t)0x7fffffff || nnz_in * (symmetrize ? 2 : 1) > (int64_t)0x7fffffff) return SC_EDOMAIN;
  if (nnz_out) *nnz_out = 0;
  struct Ctx {
    const int32_t *row, *col;
    const double* val;
    int64_t nnz, n;
    int sym;
    int64_t* rp;
    int32_t* co;
    double* vo;
    int64_t* nnz_out;
    hipStream_t st;
  } ctx{row, col, val, nnz_in, n, symmetrize ? 1 : 0, rowptr_out, col_out, val_out, nnz_out,
        reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        if (c->nnz == 0) {  // an empty list: all row pointers zero
          HIP_TRY(hipMemsetAsync(c->rp, 0, sizeof(int64_t) * (size_t)(c->n + 1), c->st));
          HIP_TRY(hipStreamSynchronize(c->st));
          return SC_OK;
        }
        const int64_t total = c->nnz * (c->sym ? 2 : 1);
        const size_t wb = coo_to_csr_workspace(total);
        DevBuf<char> work;
        DevBuf<int> bad;
        PinnedBuf<int64_t> host;
        work.alloc(wb);
        bad.alloc(1);
        host.alloc(2);
        HIP_TRY(launch_fill_int32(bad.p, 1, 0, 0, c->st));
        HIP_TRY(coo_to_csr(c->row, c->col, c->val, c->nnz, c->n, c->sym, work.p, wb, c->rp, c->co, c->vo, bad.p, c->st));
        HIP_TRY(hipMemcpyAsync(host.p, c->rp + c->n, sizeof(int64_t), hipMemcpyDeviceToHost, c->st));
        int hbad = 0;
        HIP_TRY(hipMemcpyAsync(&hbad, bad.p, sizeof(int), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        if (hbad) return SC_ECSR;
        if (c->nnz_out) *c->nnz_out = host.p[0];
        return SC_OK;
      },
      &ctx);
}

int sc_knn_search(const double* x, int64_t ldx, int64_t n, int32_t d, int32_t k_nn, int32_t* idx_out, double* dist_out,
                  void* stream) {
  if (!x || !idx_out || !dist_out || n < 0) return SC_EINVAL;
  if (d < 1 || ldx < d || n < 2 || n > (int64_t)0x7fffffff || k_nn < 1 || (int64_t)k_nn > n - 1) return SC_EDOMAIN;
  struct Ctx {
    const double* x;
    int64_t ldx, n;
    int d, k;
    int32_t* idx;
    double* dist;
    hipStream_t st;
  } ctx{x, ldx, n, d, k_nn, idx_out, dist_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        int dev = 0, lds_max = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        if (knn_search_lds_bytes(c->d, c->k) > (size_t)lds_max) return SC_EDOMAIN;  // d and k_nn too large together
        DevBuf<double> xp;
        xp.alloc((size_t)c->n * (knn_padded_dim(c->d) + 1));  // padded rows, then one squared norm per row
        HIP_TRY(launch_knn_search(c->x, c->ldx, c->n, c->d, c->k, xp.p, c->idx, c->dist, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        return SC_OK;
      },
      &ctx);
}

int sc_knn_union_pairs(const int32_t* idx, const double* dist, int64_t n, int32_t k_nn, double sigma, int32_t* edge_u,
                       int32_t* edge_v, double* val_out, int64_t* npairs_out, void* stream) {
  if (!idx || !dist || !edge_u || !edge_v || !val_out || !npairs_out || n < 0) return SC_EINVAL;
  *npairs_out = 0;
  if (k_nn < 1 || n > (int64_t)0x7fffffff || n * (int64_t)k_nn > (int64_t)0x7fffffff || sigma < 0.0 || sigma != sigma)
    return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  struct Ctx {
    const int32_t* idx;
    const double* dist;
    int64_t n;
    int k;
    double sigma;
    int32_t *eu, *ev;
    double* val;
    int64_t* np;
    hipStream_t st;
  } ctx{idx, dist, n, k_nn, sigma, edge_u, edge_v, val_out, npairs_out, reinterpret_cast<hipStream_t>(stream)};
  return guarded(
      [](void* p) {
        Ctx* c = static_cast<Ctx*>(p);
        const size_t wb = knn_pairs_workspace(c->n);
        DevBuf<char> work;
        DevBuf<int32_t> two;
        PinnedBuf<int32_t> host;
        work.alloc(wb);
        two.alloc(2);
        host.alloc(2);
        HIP_TRY(launch_knn_union_pairs(c->idx, c->dist, c->n, c->k, c->sigma, work.p, wb, c->eu, c->ev, c->val, two.p,
                                       c->st));
        HIP_TRY(hipMemcpyAsync(host.p, two.p, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->st));
        HIP_TRY(hipStreamSynchronize(c->st));
        *c->np = (int64_t)host.p[0] + (int64_t)host.p[1];
        return SC_OK;
      },
      &ctx);
}

int sc_sym_eig(const double* a, int32_t n, double* w, double* z) {
  if (!a || !w || n < 0) return SC_EINVAL;
  if (n == 0) return SC_OK;
  try {
    return sym_eig(a, n, w, z) == 0 ? SC_OK : SC_NOT_CONVERGED;
  } catch (const std::bad_alloc&) {
    return SC_ENOMEM;
  } catch (...) {
    return SC_EHIP;
  }
}

int sc_sym_eig_top(const double* a, int32_t n, int32_t count, double* w, double* z) {
  if (!a || !w || n < 0 || count < 0 || (count > 0 && !z)) return SC_EINVAL;
  if (count > n) return SC_EDOMAIN;
  if (n == 0) return SC_OK;
  try {
    SelectedEig se;
    if (se.factor(a, n) != 0) return SC_NOT_CONVERGED;
    std::memcpy(w, se.values().data(), sizeof(double) * n);
    std::vector<int> idx(count);
    for (int t = 0; t < count; ++t) idx[t] = n - 1 - t;
    se.vectors(idx.data(), count, z);
    return SC_OK;
  } catch (const std::bad_alloc&) {
    return SC_ENOMEM;
  } catch (...) {
    return SC_EHIP;
  }
}

}  // extern "C"
