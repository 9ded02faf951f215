// Host-side dense symmetric eigensolver used for the projected Lanczos problem.
#pragma once

namespace sceig {

// All eigenpairs of the symmetric n x n matrix a (row-major, both triangles filled; only read).
// w[n]: eigenvalues ascending.  z (n x n row-major, may be null): column t is the eigenvector of w[t].
// Returns 0 on success, 1 if the QL iteration did not converge.
int sym_eig(const double* a, int n, double* w, double* z);

}  // namespace sceig
