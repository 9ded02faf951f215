// Dense symmetric eigensolver for the projected Lanczos problem (the m x m eigendecomposition
// of the paper's Section IV-B complexity discussion).  Host code, no GPU, no external LAPACK.
//
// Method (textbook): Householder reduction to tridiagonal form, accumulation of the orthogonal
// factor, implicit QL iteration with Wilkinson shifts.  The plane rotations of one QL sweep are
// recorded and then applied to all rows of the eigenvector matrix at once, which makes the
// O(n^3) part row-parallel (OpenMP) and contiguous in memory.
#include "sym_eig.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

#include <omp.h>

namespace sceig {

namespace {

constexpr int kParallelMin = 256;  // below this size the OpenMP fork/join costs more than it saves

// Reduce the symmetric matrix held in q (row-major n x n, full storage) to tridiagonal form
// (diagonal d, sub-diagonal e with e[i] coupling i and i+1) and overwrite q with the orthogonal
// matrix Q such that A = Q T Q^T.
void tridiagonalize(int n, std::vector<double>& q, std::vector<double>& d, std::vector<double>& e,
                    std::vector<double>& vs, std::vector<double>& betas, bool form_q) {
  vs.assign((size_t)n * n, 0.0);  // Householder vectors, vector k in row k (entries k+1..n-1)
  betas.assign(n, 0.0);
  std::vector<double> p(n), w(n), scatter;
  double* a = q.data();
  for (int k = 0; k + 2 < n; ++k) {
    // x = A[k+1:n, k]
    double* v = &vs[(size_t)k * n];
    double xnorm2 = 0.0;
    for (int i = k + 2; i < n; ++i) xnorm2 += a[(size_t)i * n + k] * a[(size_t)i * n + k];
    const double x0 = a[(size_t)(k + 1) * n + k];
    if (xnorm2 == 0.0) {
      betas[k] = 0.0;  // already tridiagonal in this column
      e[k] = x0;
      d[k] = a[(size_t)k * n + k];
      continue;
    }
    const double alpha = -std::copysign(std::sqrt(x0 * x0 + xnorm2), x0);
    // v = x - alpha e1, normalised so that v[0] = 1
    const double v0 = x0 - alpha;
    v[k + 1] = 1.0;
    for (int i = k + 2; i < n; ++i) v[i] = a[(size_t)i * n + k] / v0;
    const double beta = -v0 / alpha;  // H = I - beta v v^T
    betas[k] = beta;
    e[k] = alpha;
    d[k] = a[(size_t)k * n + k];
    // p = beta * A22 v and A22 -= v w^T + w v^T, both on the lower triangle only (row i, columns lo..i)
    const int lo = k + 1;
    const int len = n - lo;
    if (len >= kParallelMin) {
      // rows are dealt out cyclically in chunks (a fixed assignment, so the result does not depend on timing);
      // every thread scatters into a buffer of its own and the buffers are added in thread order
      const int nth = omp_get_max_threads();
      if ((int)scatter.size() < nth * n) scatter.resize((size_t)nth * n);
#pragma omp parallel num_threads(nth)
      {
        double* pp = scatter.data() + (size_t)omp_get_thread_num() * n;
        for (int j = lo; j < n; ++j) pp[j] = 0.0;
#pragma omp for schedule(static, 8)
        for (int i = lo; i < n; ++i) {
          const double* row = a + (size_t)i * n;
          const double vi = v[i];
          double s = 0.0;
#pragma omp simd reduction(+ : s)
          for (int j = lo; j < i; ++j) {
            s += row[j] * v[j];
            pp[j] += row[j] * vi;
          }
          pp[i] += s + row[i] * vi;
        }
      }
      for (int j = lo; j < n; ++j) {
        double tot = 0.0;
        for (int t = 0; t < nth; ++t) tot += scatter[(size_t)t * n + j];
        p[j] = beta * tot;
      }
    } else {
      for (int i = lo; i < n; ++i) p[i] = 0.0;
      for (int i = lo; i < n; ++i) {
        const double* row = a + (size_t)i * n;
        const double vi = v[i];
        double s = 0.0;
        double* pp = p.data();
#pragma omp simd reduction(+ : s)
        for (int j = lo; j < i; ++j) {
          s += row[j] * v[j];
          pp[j] += row[j] * vi;
        }
        p[i] += s + row[i] * vi;
      }
      for (int i = lo; i < n; ++i) p[i] *= beta;
    }
    double pv = 0.0;
    for (int i = lo; i < n; ++i) pv += p[i] * v[i];
    const double half = 0.5 * beta * pv;
    for (int i = lo; i < n; ++i) w[i] = p[i] - half * v[i];
#pragma omp parallel for schedule(static, 8) if (len >= kParallelMin)
    for (int i = lo; i < n; ++i) {
      double* row = a + (size_t)i * n;
      const double vi = v[i], wi = w[i];
      const double* wp = w.data();
#pragma omp simd
      for (int j = lo; j <= i; ++j) row[j] -= vi * wp[j] + wi * v[j];
    }
  }
  if (n >= 2) {
    d[n - 2] = a[(size_t)(n - 2) * n + (n - 2)];
    e[n - 2] = a[(size_t)(n - 1) * n + (n - 2)];
  }
  d[n - 1] = a[(size_t)(n - 1) * n + (n - 1)];
  if (n >= 1) e[n - 1] = 0.0;
  if (!form_q) return;
  // Q = H_0 H_1 ... H_{n-3}, accumulated backwards into q (row-major)
  std::fill(q.begin(), q.end(), 0.0);
  for (int i = 0; i < n; ++i) a[(size_t)i * n + i] = 1.0;
  std::vector<double> t(n);
  for (int k = n - 3; k >= 0; --k) {
    const double beta = betas[k];
    if (beta == 0.0) continue;
    const double* v = &vs[(size_t)k * n];
    const int lo = k + 1;
    // Q[lo:, lo:] -= beta v (v^T Q[lo:, lo:])
    std::fill(t.begin(), t.end(), 0.0);
    for (int i = lo; i < n; ++i) {
      const double vi = v[i];
      const double* row = a + (size_t)i * n;
      for (int j = lo; j < n; ++j) t[j] += vi * row[j];
    }
#pragma omp parallel for schedule(static) if (n - lo >= kParallelMin)
    for (int i = lo; i < n; ++i) {
      const double bv = beta * v[i];
      double* row = a + (size_t)i * n;
      for (int j = lo; j < n; ++j) row[j] -= bv * t[j];
    }
  }
}

struct Rot {
  double c, s;
};

// Implicit QL on (d, e); z (row-major n x n, may be null) is multiplied from the right by the
// accumulated rotations.  Returns false if some eigenvalue needs more than 60 iterations.
template <typename Record>
bool ql_implicit(int n, std::vector<double>& d, std::vector<double>& e, double* z, Record record) {
  std::vector<Rot> rots(n);
  for (int l = 0; l < n; ++l) {
    int iter = 0;
    while (true) {
      int m = l;
      for (; m + 1 < n; ++m) {
        const double dd = std::fabs(d[m]) + std::fabs(d[m + 1]);
        if (std::fabs(e[m]) <= 2.220446049250313e-16 * dd) break;
      }
      if (m == l) break;
      if (++iter > 60) return false;
      // Wilkinson shift from the leading 2x2 of the unreduced block
      double g = (d[l + 1] - d[l]) / (2.0 * e[l]);
      double r = std::hypot(g, 1.0);
      g = d[m] - d[l] + e[l] / (g + std::copysign(r, g));
      double s = 1.0, c = 1.0, p = 0.0;
      int i = m - 1;
      bool underflow = false;
      for (; i >= l; --i) {
        double f = s * e[i];
        const double b = c * e[i];
        r = std::sqrt(f * f + g * g);  // entries are O(1): no overflow; an underflow to 0 is handled below
        e[i + 1] = r;
        if (r == 0.0) {
          d[i + 1] -= p;
          e[m] = 0.0;
          underflow = true;
          break;
        }
        s = f / r;
        c = g / r;
        g = d[i + 1] - p;
        r = (d[i] - g) * s + 2.0 * c * b;
        p = s * r;
        d[i + 1] = g + p;
        g = c * r - b;
        rots[i] = {c, s};
      }
      const int first = underflow ? i + 1 : l;  // rotations recorded for indices first..m-1
      for (int t = m - 1; t >= first; --t) record(t, rots[t].c, rots[t].s);
      if (z) {
        const int cnt = m - first;
        if (cnt > 0) {
#pragma omp parallel for schedule(static) if (n >= kParallelMin && (long)n * cnt >= 20000)
          for (int row = 0; row < n; ++row) {
            double* zr = z + (size_t)row * n;
            for (int t = m - 1; t >= first; --t) {
              const double cc = rots[t].c, ss = rots[t].s;
              const double f = zr[t + 1];
              zr[t + 1] = ss * zr[t] + cc * f;
              zr[t] = cc * zr[t] - ss * f;
            }
          }
        }
      }
      if (underflow) continue;
      d[l] -= p;
      e[l] = g;
      e[m] = 0.0;
    }
  }
  return true;
}

}  // namespace

int sym_eig(const double* a_in, int n, double* w, double* z_out) {
  if (n <= 0) return 0;
  std::vector<double> q((size_t)n * n);
  // symmetrise on the way in (callers fill both triangles, this removes rounding asymmetry)
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < n; ++j) q[(size_t)i * n + j] = 0.5 * (a_in[(size_t)i * n + j] + a_in[(size_t)j * n + i]);
  std::vector<double> d(n), e(n);
  if (n == 1) {
    w[0] = q[0];
    if (z_out) z_out[0] = 1.0;
    return 0;
  }
  std::vector<double> vs, betas;
  tridiagonalize(n, q, d, e, vs, betas, z_out != nullptr);
  if (!ql_implicit(n, d, e, z_out ? q.data() : nullptr, [](int, double, double) {})) return 1;
  // sort ascending, permuting eigenvector columns
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return d[x] < d[y]; });
  for (int t = 0; t < n; ++t) w[t] = d[order[t]];
  if (z_out) {
#pragma omp parallel for schedule(static) if (n >= kParallelMin)
    for (int i = 0; i < n; ++i) {
      const double* src = &q[(size_t)i * n];
      double* dst = z_out + (size_t)i * n;
      for (int t = 0; t < n; ++t) dst[t] = src[order[t]];
    }
  }
  return 0;
}

int SelectedEig::factor(const double* a_in, int n) {
  n_ = n;
  w_.assign(n, 0.0);
  order_.resize(n);
  rots_.clear();
  if (n <= 0) return 0;
  std::vector<double> q((size_t)n * n);
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < n; ++j) q[(size_t)i * n + j] = 0.5 * (a_in[(size_t)i * n + j] + a_in[(size_t)j * n + i]);
  std::vector<double> d(n), e(n);
  if (n == 1) {
    w_[0] = q[0];
    order_[0] = 0;
    vs_.assign(1, 0.0);
    betas_.assign(1, 0.0);
    return 0;
  }
  tridiagonalize(n, q, d, e, vs_, betas_, false);
  rots_.reserve((size_t)n * n);
  if (!ql_implicit(n, d, e, nullptr, [this](int i, double c, double s) { rots_.push_back(Rot{i, c, s}); })) return 1;
  std::iota(order_.begin(), order_.end(), 0);
  std::stable_sort(order_.begin(), order_.end(), [&](int x, int y) { return d[x] < d[y]; });
  for (int t = 0; t < n; ++t) w_[t] = d[order_[t]];
  return 0;
}

void SelectedEig::vectors(const int* idx, int count, double* out) const {
  const int n = n_;
  if (n <= 0 || count <= 0) return;
  // Eigenvectors of the tridiagonal matrix: Z e_j = G_1 (G_2 (... (G_N e_j))), so the recorded rotations are replayed
  // backwards on the selected unit vectors; then back through the reflectors: Y = H_0 H_1 ... H_{n-3} Z.  Columns are
  // independent.  Every thread takes a slice of them into a buffer of its own (n x width, contiguous) and copies the
  // result back at the end: slices of one shared array would put several threads on the same cache lines for every
  // one of the ~n^2 rotations.
  const int slices = (count >= 32 && (long)n * count >= 20000) ? std::min(omp_get_max_threads(), count / 8) : 1;
#pragma omp parallel for schedule(static) num_threads(slices) if (slices > 1)
  for (int sl = 0; sl < slices; ++sl) {
    const int t0 = (int)((long)count * sl / slices), t1 = (int)((long)count * (sl + 1) / slices);
    const int w = t1 - t0;
    if (w <= 0) continue;
    std::vector<double> buf((size_t)n * w, 0.0), tmp(w);
    for (int t = t0; t < t1; ++t) buf[(size_t)order_[idx[t]] * w + (t - t0)] = 1.0;
    for (size_t r = rots_.size(); r-- > 0;) {
      const Rot& g = rots_[r];
      double* a = buf.data() + (size_t)g.i * w;
      double* b = a + w;
      const double c = g.c, s = g.s;
#pragma omp simd
      for (int t = 0; t < w; ++t) {
        const double x = a[t], y = b[t];
        a[t] = c * x + s * y;
        b[t] = c * y - s * x;
      }
    }
    for (int k = n - 3; k >= 0; --k) {
      const double beta = betas_[k];
      if (beta == 0.0) continue;
      const double* v = &vs_[(size_t)k * n];
      for (int t = 0; t < w; ++t) tmp[t] = 0.0;
      for (int i = k + 1; i < n; ++i) {
        const double vi = v[i];
        const double* row = buf.data() + (size_t)i * w;
#pragma omp simd
        for (int t = 0; t < w; ++t) tmp[t] += vi * row[t];
      }
      for (int i = k + 1; i < n; ++i) {
        const double bv = beta * v[i];
        double* row = buf.data() + (size_t)i * w;
#pragma omp simd
        for (int t = 0; t < w; ++t) row[t] -= bv * tmp[t];
      }
    }
    for (int i = 0; i < n; ++i) std::memcpy(out + (size_t)i * count + t0, buf.data() + (size_t)i * w, sizeof(double) * w);
  }
}

}  // namespace sceig
