// Offline host SVD used by rsparse_prepare (R-Sparse, Sec. 3.4: the low-rank factors come from
// one SVD of the pretrained weight, computed offline).  Plain C++, no BLAS/LAPACK.
#pragma once
#include <cstddef>

namespace rsparse {

// Top-r singular triplets of W [m][n] row-major (m = d_out, n = d_in), r <= min(m, n):
// U [m][r] (orthonormal columns), S [r] descending, V [n][r] (orthonormal columns), so that
// W ~ U diag(S) V^T is the best rank-r approximation.  Block subspace iteration on a
// (2r+16)-dimensional block until the Ritz values settle, then a Jacobi eigensolve of the
// small projected Gram matrix.  Deterministic (fixed seed).  Returns 0, or -1 with a message.
int svd_top_r(const double *W, int m, int n, int r, double *U, double *S, double *V, char *msg,
              size_t msglen);

}  // namespace rsparse
