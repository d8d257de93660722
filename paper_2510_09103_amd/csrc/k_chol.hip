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

// R <- C^-1 R on 64 whole columns, or L <- L C on 64 whole rows, in place (fp64 products, fp32 stores): the r x 64
// result Out[a][j] = sum_k M[k][a] T[k][j] with T the tile of the factor (contraction index k = row of R / column of
// L) and M[k][a] = C^-1[a][k] (for R) or C[k][a] (for L).  The whole tile goes to LDS first (fp32, as stored), so the
// workgroup may overwrite its columns / rows afterwards; M is staged 32 values of k at a time (fp64).  A thread owns
// two 4 x 4 pieces of the result: per k one 16-byte read of T and two of M feed 16 multiply-adds.  Entries of the
// triangular matrices outside the triangle are exact zeros; a thread skips the slabs of k that lie wholly outside
// its piece's part of the triangle.
constexpr int RG_W = 64;                 // columns of R / rows of L per workgroup
constexpr int RG_K = 32;                 // values of the contraction index per staged slab of M
constexpr int RG_MS = 128 + 2;           // LDS row stride of M (doubles): rows stay 16-byte aligned
__global__ __launch_bounds__(256) void regauge_apply_kernel(const RegaugeItem* __restrict__ items, Bases b) {
  __shared__ __attribute__((aligned(16))) float T[128 * RG_W];        // T[k][j]
  __shared__ __attribute__((aligned(16))) double Ms[RG_K * RG_MS];    // Ms[kk][a] = M[k0 + kk][a], zero for a >= r
  const RegaugeItem it = items[blockIdx.x];
  const int r = it.r, tid = threadIdx.x;
  float* X = reinterpret_cast<float*>(b.state + it.off_x);
  const double* __restrict__ Cm = reinterpret_cast<const double*>(b.ws + it.off_c);
  const int width = it.len - it.first < RG_W ? it.len - it.first : RG_W;
  const bool isL = it.is_L != 0;
  if (!isL) {
    for (int e = tid; e < r * RG_W; e += 256) {
      const int k = e / RG_W, j = e % RG_W;
      T[e] = j < width ? X[(int64_t)k * it.len + it.first + j] : 0.f;
    }
  } else {
    for (int e = tid; e < r * RG_W; e += 256) {
      const int j = e / r, k = e % r;                 // row j of the 64, column k of L: contiguous in memory along k
      T[k * RG_W + j] = j < width ? X[(int64_t)(it.first + j) * r + k] : 0.f;
    }
  }
  // this thread's two pieces: values a0 .. a0+3 of the free index, positions j0 .. j0+3.  R: consecutive lanes walk
  // along j (their stores are contiguous along a row of R); L: along a (contiguous along a row of L).
  int a0[2], j0[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int q = tid + 256 * u;
    a0[u] = 4 * (isL ? q % 32 : q / 16);
    j0[u] = 4 * (isL ? q / 32 : q % 16);
  }
  double acc[2][4][4];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) acc[u][x][y] = 0.0;
  for (int k0 = 0; k0 < r; k0 += RG_K) {
    __syncthreads();                                  // the tile is in LDS / the previous slab has been used
    for (int e = tid; e < RG_K * 128; e += 256) {
      int kk, a;
      if (isL) { kk = e / 128; a = e % 128; } else { a = e / RG_K; kk = e % RG_K; }   // contiguous in memory either way
      const int k = k0 + kk;
      double v = 0.0;
      if (k < r && a < r) v = isL ? Cm[(int64_t)k * r + a] : Cm[(int64_t)a * r + k];
      Ms[kk * RG_MS + a] = v;
    }
    __syncthreads();
    const int kn = r - k0 < RG_K ? r - k0 : RG_K;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      // R: M[k][a] != 0 only for k <= a; L: only for k >= a
      const bool live = a0[u] < r && (isL ? k0 + RG_K > a0[u] : k0 <= a0[u] + 3);
      if (!live) continue;
      for (int kk = 0; kk < kn; ++kk) {
        const float4 t4 = *reinterpret_cast<const float4*>(&T[(k0 + kk) * RG_W + j0[u]]);
        const double2 m01 = *reinterpret_cast<const double2*>(&Ms[kk * RG_MS + a0[u]]);
        const double2 m23 = *reinterpret_cast<const double2*>(&Ms[kk * RG_MS + a0[u] + 2]);
        const double tv[4] = {(double)t4.x, (double)t4.y, (double)t4.z, (double)t4.w};
        const double mv[4] = {m01.x, m01.y, m23.x, m23.y};
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int y = 0; y < 4; ++y) acc[u][x][y] = fma(mv[x], tv[y], acc[u][x][y]);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int a = a0[u] + x;
      if (a >= r) continue;
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int j = j0[u] + y;
        if (j >= width) continue;
        if (isL) X[(int64_t)(it.first + j) * r + a] = (float)acc[u][x][y];
        else X[(int64_t)a * it.len + it.first + j] = (float)acc[u][x][y];
      }
    }
  }
}

}  // namespace

void launch_regauge_apply(const RegaugeItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(regauge_apply_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

void launch_chol(const CholItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(chol_inv_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

}  // namespace adapm
