// Host-side dense symmetric eigensolver used for the projected Lanczos problem.
#pragma once

#include <vector>

namespace sceig {

// All eigenpairs of the symmetric n x n matrix a (row-major, both triangles filled; only read).
// w[n]: eigenvalues ascending.  z (n x n row-major, may be null): column t is the eigenvector of w[t].
// Returns 0 on success, 1 if the QL iteration did not converge.
int sym_eig(const double* a, int n, double* w, double* z);

// Same factorisation, but eigenvectors are produced only for the eigenvalues asked for: the plane rotations of
// the QL iteration are recorded and replayed backwards on the selected unit vectors, which are then taken back
// through the Householder reflectors.  Cost ~ 4/3 n^3 + O(n^2 * count) instead of ~ 9 n^3.
class SelectedEig {
 public:
  // Factorises a (n x n, row-major, symmetric).  Returns 0, or 1 if QL did not converge.
  int factor(const double* a, int n);
  int size() const { return n_; }
  // Eigenvalues in ascending order.
  const std::vector<double>& values() const { return w_; }
  // out (n x count, row-major): column t is the unit eigenvector of values()[idx[t]].
  void vectors(const int* idx, int count, double* out) const;

 private:
  struct Rot {
    int i;
    double c, s;
  };
  int n_ = 0;
  std::vector<double> w_;        // ascending
  std::vector<int> order_;       // order_[t] = position in the QL output of the t-th smallest eigenvalue
  std::vector<double> vs_;       // Householder vectors (row k: entries k+1..n-1)
  std::vector<double> betas_;
  std::vector<Rot> rots_;
};

}  // namespace sceig
