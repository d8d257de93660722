// fp64 Cholesky factorisation and triangular inverse of the r x r Gram matrix R R^T.
// Used after Alg. 2 when the refresh period T exceeds 1: with R R^T = C C^T the factors are
// re-expressed as (L C, C^-1 R), which keeps the product L R and makes the rows of R
// orthonormal, so that the least-squares fit of L with R held is a plain projection.
// One workgroup per low-rank block (r <= 128: the matrix stays in LDS); fp64 keeps the orthonormality error at fp32 rounding
// level whatever the conditioning of R.
// A Gram matrix that is not positive definite in fp64 (a pivot that is zero, negative or not finite: R has lost
// rank, e.g. factors that are exactly zero) has no such factorisation; the kernel then writes C = C^-1 = I, so that
// the block's (L, R) pass through the re-expression unchanged instead of turning into NaN.
#include "adapm_plan.h"

namespace adapm {

namespace {

// r above CH_MAX: in place in global memory
__device__ void chol_inv_global(double* A, double* X, int r) {
  const int tid = threadIdx.x;
  bool bad = false;
  // right-looking Cholesky, lower triangle, in place
  for (int j = 0; j < r; ++j) {
    const double piv = A[(int64_t)j * r + j];        // the same value in every thread
    if (!(piv > 0.0) || !isfinite(piv)) { bad = true; break; }
    const double d = sqrt(piv);
    __syncthreads();
    for (int i = j + tid; i < r; i += 256) A[(int64_t)i * r + j] = (i == j) ? d : A[(int64_t)i * r + j] / d;
    __syncthreads();
    const int rem = r - j - 1;                       // trailing rows j+1 .. r-1
    for (int64_t e = tid; e < (int64_t)rem * rem; e += 256) {
      const int i = j + 1 + (int)(e / rem), k = j + 1 + (int)(e % rem);
      if (k <= i) A[(int64_t)i * r + k] -= A[(int64_t)i * r + j] * A[(int64_t)k * r + j];
    }
    __syncthreads();
  }
  __syncthreads();
  if (bad) {
    for (int64_t e = tid; e < (int64_t)r * r; e += 256) A[e] = X[e] = (e / r == e % r) ? 1.0 : 0.0;
    return;
  }
  for (int64_t e = tid; e < (int64_t)r * r; e += 256) {
    const int i = (int)(e / r), k = (int)(e % r);
    if (k > i) A[e] = 0.0;
  }
  __syncthreads();
  // X = C^-1 by forward substitution, one column per thread
  for (int j = tid; j < r; j += 256) {
    for (int a = 0; a < r; ++a) {
      double s = (a == j) ? 1.0 : 0.0;
      if (a < j) { X[(int64_t)a * r + j] = 0.0; continue; }
      for (int c = j; c < a; ++c) s -= A[(int64_t)a * r + c] * X[(int64_t)c * r + j];
      X[(int64_t)a * r + j] = s / A[(int64_t)a * r + a];
    }
  }
}

constexpr int CH_MAX = 128;   // largest r factorised in LDS (every block of the MFMA path)

// The same operations in the same order with the matrix in LDS: C in the lower triangle, the strictly
// lower part of C^-1 transposed into the (otherwise unused) upper triangle, its diagonal beside it.
__global__ __launch_bounds__(256) void chol_inv_kernel(const CholItem* __restrict__ items, Bases b) {
  __shared__ double S[CH_MAX * (CH_MAX + 1)];
  __shared__ double xd[CH_MAX];
  const CholItem it = items[blockIdx.x];
  const int r = it.r, tid = threadIdx.x;
  double* A = reinterpret_cast<double*>(b.ws + it.off_gram);
  double* X = reinterpret_cast<double*>(b.ws + it.off_inv);
  if (r > CH_MAX) { chol_inv_global(A, X, r); return; }
  const int ld = r | 1;                              // odd row stride: a column walks through all banks
  for (int e = tid; e < r * r; e += 256) S[(e / r) * ld + e % r] = A[e];
  __syncthreads();
  const int tx = tid & 15, ty = tid >> 4;
  bool bad = false;
  for (int j = 0; j < r; ++j) {
    const double piv = S[j * ld + j];                // the same value in every thread
    if (!(piv > 0.0) || !isfinite(piv)) { bad = true; break; }
    const double d = sqrt(piv);
    __syncthreads();
    for (int i = j + tid; i < r; i += 256) S[i * ld + j] = (i == j) ? d : S[i * ld + j] / d;
    __syncthreads();
    for (int i = j + 1 + ty; i < r; i += 16) {
      const double lij = S[i * ld + j];
      for (int k = j + 1 + tx; k <= i; k += 16) S[i * ld + k] -= lij * S[k * ld + j];
    }
    __syncthreads();
  }
  if (bad) {                                         // uniform: every thread saw the same pivot
    for (int e = tid; e < r * r; e += 256) A[e] = X[e] = (e / r == e % r) ? 1.0 : 0.0;
    return;
  }
  // column j of C^-1 by forward substitution, one column per thread; thread j writes row j of the upper
  // triangle and xd[j] only, and reads nothing another thread writes
  if (tid < r) {
    const int j = tid;
    for (int a = j; a < r; ++a) {
      double s = (a == j) ? 1.0 : 0.0;
      for (int c = j; c < a; ++c) s -= S[a * ld + c] * (c == j ? xd[j] : S[j * ld + c]);
      const double x = s / S[a * ld + a];
      if (a == j) xd[j] = x; else S[j * ld + a] = x;
    }
  }
  __syncthreads();
  for (int e = tid; e < r * r; e += 256) {
    const int i = e / r, k = e % r;
    A[e] = k <= i ? S[i * ld + k] : 0.0;
    X[e] = k < i ? S[k * ld + i] : (k == i ? xd[i] : 0.0);
  }
}

}  // namespace

void launch_chol(const CholItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(chol_inv_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

}  // namespace adapm
