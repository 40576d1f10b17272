// Small dense kernel of the RSVD compressor (Experimental Setup: randomized SVD of Halko et al.): the
// triangular factor of a k x k Gram matrix and its inverse, the middle step of a Cholesky QR.  The large
// products around it (X.Omega, Yr^T.Yr, Yr.R^-1, X^T.U, U^T.dY) run on the generic MFMA kernels.
#pragma once
#include "acc_common.h"

namespace acc {

constexpr int kRsvdMaxRank = 128;  // k x k doubles must fit the 160 KB of LDS

// G [k, k] (symmetric positive semi-definite, fp32) -> Rinv [k, k] fp32 with G = R^T R, R upper
// triangular with positive diagonal, Rinv = R^-1 (upper triangular).  One work-group, fp64 inside.
// A pivot that is not positive beyond rounding (column j of the factored matrix depends on the earlier
// ones) is dropped: row and column j of Rinv are zero, so the corresponding basis vector comes out as
// zero and the span of the others is unchanged.
// Dynamic LDS: k * k doubles.
__global__ __launch_bounds__(256) void chol_inverse_kernel(const float* __restrict__ G, float* __restrict__ Rinv,
                                                           int k) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  double* A = (double*)smem_raw;  // [k][k]; the upper triangle becomes R
  __shared__ double s_maxdiag;
  __shared__ int s_dead[kRsvdMaxRank];
  const int tid = threadIdx.x;
  for (int e = tid; e < k * k; e += 256) A[e] = (double)G[e];
  __syncthreads();
  if (tid == 0) {
    double m = 0.0;
    for (int j = 0; j < k; ++j) m = A[j * k + j] > m ? A[j * k + j] : m;
    s_maxdiag = m;
  }
  __syncthreads();
  const double tol = s_maxdiag * 1e-6;  // fp32 Gram: entries carry ~1e-7 relative rounding
  for (int j = 0; j < k; ++j) {
    const double piv = A[j * k + j];
    const bool dead = !(piv > tol);
    __syncthreads();  // everyone has read the pivot before row j is scaled
    if (tid == 0) s_dead[j] = dead ? 1 : 0;
    const double inv_d = dead ? 0.0 : 1.0 / sqrt(piv);
    for (int c = j + tid; c < k; c += 256) A[j * k + c] = dead ? 0.0 : A[j * k + c] * inv_d;  // R[j][c]
    __syncthreads();
    const int m = k - j - 1;  // trailing (m x m) update, upper triangle only
    for (int e = tid; e < m * m; e += 256) {
      const int i = j + 1 + e / m, c = j + 1 + e % m;
      if (c >= i) A[i * k + c] -= A[j * k + i] * A[j * k + c];
    }
    __syncthreads();
  }
  // Back substitution, one column of the inverse per thread: R x = e_c, x[i] = 0 for i > c.
  // Dropped pivots give x[j] = 0 and an all-zero column j.
  for (int c = tid; c < k; c += 256) {
    double x[kRsvdMaxRank];
    for (int i = c; i >= 0; --i) {
      double s = (i == c) ? 1.0 : 0.0;
      for (int t = i + 1; t <= c; ++t) s -= A[i * k + t] * x[t];
      x[i] = (s_dead[i] || s_dead[c]) ? 0.0 : s / A[i * k + i];
    }
    for (int i = 0; i < k; ++i) Rinv[i * k + c] = (i <= c) ? (float)x[i] : 0.f;
  }
}

}  // namespace acc
