// fp64-accumulate strided two-product GEMM on the vector ALUs (the "F64" contraction mode):
//   Out = a1 * A1 B1 + a2 * A2 B2 + g * X + d * Y
// One launch covers a list of 64 x 64 output tiles drawn from many independent problems,
// so every thin product of Alg. 2 (G R^T, L^T G, the four r x r Gram matrices, the factor
// updates, the reconstruction L_{t-1}R_{t-1} - L_t R_t) of every low-rank block runs in a
// handful of launches.  Operands (bf16 / fp32 / fp64) convert exactly to fp64; sums run in
// ascending k, so results are deterministic.
#include "adapm_plan.h"

namespace adapm {

namespace {

constexpr int TM = 64, TN = 64, TK = 16, PAD = 2;

__device__ __forceinline__ double load_el(const char* base, int dtype, int64_t idx) {
  if (dtype == DT_F32) return (double)reinterpret_cast<const float*>(base)[idx];
  if (dtype == DT_BF16) return (double)__uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx]) << 16);
  return reinterpret_cast<const double*>(base)[idx];
}

// Four elements of an operand tile per thread.  Every load is issued unconditionally on a clamped (always
// valid) index and masked afterwards: a load inside its own bounds check would wait for the previous one.
template <int DT>
__device__ __forceinline__ void fetch4_t(const char* base, const int64_t (&idx)[4], const bool (&ok)[4], double (&x)[4]) {
  if (DT == DT_F32) {
    float r[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) r[p] = reinterpret_cast<const float*>(base)[ok[p] ? idx[p] : 0];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = ok[p] ? (double)r[p] : 0.0;
  } else if (DT == DT_BF16) {
    uint16_t r[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) r[p] = reinterpret_cast<const uint16_t*>(base)[ok[p] ? idx[p] : 0];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = ok[p] ? (double)__uint_as_float(((uint32_t)r[p]) << 16) : 0.0;
  } else {
    double r[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) r[p] = reinterpret_cast<const double*>(base)[ok[p] ? idx[p] : 0];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = ok[p] ? r[p] : 0.0;
  }
}
__device__ __forceinline__ void fetch4(const char* base, int dtype, const int64_t (&idx)[4], const bool (&ok)[4], double (&x)[4]) {
  if (dtype == DT_F32) fetch4_t<DT_F32>(base, idx, ok, x);
  else if (dtype == DT_BF16) fetch4_t<DT_BF16>(base, idx, ok, x);
  else fetch4_t<DT_F64>(base, idx, ok, x);
}

// contraction over k in [kbeg, K)
__device__ __forceinline__ void product(const Mat& A, const Mat& B, int M, int N, int kbeg, int K, int i0, int j0,
                                        const Bases& bs, double (*As)[TM + PAD], double (*Bs)[TN + PAD],
                                        double acc[4][4]) {
  const char* Ab = resolve(A.ref, bs);
  const char* Bb = resolve(B.ref, bs);
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const bool a_kfast = (A.s1 == 1), b_jfast = (B.s1 == 1);
  int ia[4], ka[4], jb[4], kb[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int idx = tid + p * 256;
    if (a_kfast) { ka[p] = idx & 15; ia[p] = idx >> 4; } else { ia[p] = idx & 63; ka[p] = idx >> 6; }
    if (b_jfast) { jb[p] = idx & 63; kb[p] = idx >> 6; } else { kb[p] = idx & 15; jb[p] = idx >> 4; }
  }
  auto fetch = [&](int k0, double (&xa)[4], double (&xb)[4]) {
    int64_t ix[4];
    bool ok[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      ok[p] = i0 + ia[p] < M && k0 + ka[p] < K;
      ix[p] = (int64_t)(i0 + ia[p]) * A.s0 + (int64_t)(k0 + ka[p]) * A.s1;
    }
    fetch4(Ab, A.dtype, ix, ok, xa);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      ok[p] = j0 + jb[p] < N && k0 + kb[p] < K;
      ix[p] = (int64_t)(k0 + kb[p]) * B.s0 + (int64_t)(j0 + jb[p]) * B.s1;
    }
    fetch4(Bb, B.dtype, ix, ok, xb);
  };
  double xa[4], xb[4];
  fetch(kbeg, xa, xb);
  for (int k0 = kbeg; k0 < K; k0 += TK) {
#pragma unroll
    for (int p = 0; p < 4; ++p) { As[ka[p]][ia[p]] = xa[p]; Bs[kb[p]][jb[p]] = xb[p]; }
    __syncthreads();
    if (k0 + TK < K) fetch(k0 + TK, xa, xb);       // the next chunk travels while this one is multiplied
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      double a[4], b[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { a[q] = As[kk][ty * 4 + q]; b[q] = Bs[kk][tx * 4 + q]; }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[q][c] = fma(a[q], b[c], acc[q][c]);
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void gemm64_kernel(const GemmProblem* __restrict__ probs,
                                                     const GemmTile* __restrict__ tiles, Bases bs) {
  __shared__ double As[TK][TM + PAD];
  __shared__ double Bs[TK][TN + PAD];
  const GemmTile t = tiles[blockIdx.x];
  const GemmProblem& P = probs[t.prob];
  const int i0 = t.ti * TM, j0 = t.tj * TN;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  double acc[4][4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[q][c] = 0.0;
  if (P.K1 > 0) {
    // a lower-triangular operand of the first product (tri = 1: A1, tri = 2: B1) leaves part of the contraction
    // identically zero for this tile: rows i0 .. i0+63 of A1 end at column i0+63, columns j0 .. of B1 start at row j0
    const int ke = P.tri == 1 ? (P.K1 < i0 + TM ? P.K1 : i0 + TM) : P.K1;
    const int kb = P.tri == 2 ? (j0 / TK) * TK : 0;
    product(P.A1, P.B1, P.M, P.N, kb, ke, i0, j0, bs, As, Bs, acc);
    const double a1 = P.a1 * (P.scale_g ? (double)grad_scale(bs) : 1.0);   // the gradient enters clipped
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[q][c] *= a1;
  }
  if (P.K2 > 0) {
    double acc2[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc2[q][c] = 0.0;
    product(P.A2, P.B2, P.M, P.N, 0, P.K2, i0, j0, bs, As, Bs, acc2);
    const double a2 = P.a2;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int c = 0; c < 4; ++c) acc[q][c] = fma(a2, acc2[q][c], acc[q][c]);
  }
  const char* Xb = P.X.ref.space != SP_NONE ? resolve(P.X.ref, bs) : nullptr;
  const char* Yb = P.Y.ref.space != SP_NONE ? resolve(P.Y.ref, bs) : nullptr;
  char* Ob = resolve(P.Out.ref, bs);
  // optional device scalar on everything but X (normalised step of Alg. 2)
  const double step_scale = P.off_s >= 0 ? *reinterpret_cast<const double*>(bs.ws + P.off_s) : 1.0;
  // X and Y are read unconditionally on clamped indices (independent loads); the bounds check guards the store
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int i = i0 + ty * 4 + q;
    const int ic = i < P.M ? i : 0;
    double xv[4] = {0.0, 0.0, 0.0, 0.0}, yv[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = j0 + tx * 4 + c;
      const int jc = j < P.N ? j : 0;
      if (Xb) xv[c] = load_el(Xb, P.X.dtype, (int64_t)ic * P.X.s0 + (int64_t)jc * P.X.s1);
      if (Yb) yv[c] = load_el(Yb, P.Y.dtype, (int64_t)ic * P.Y.s0 + (int64_t)jc * P.Y.s1);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = j0 + tx * 4 + c;
      if (i >= P.M || j >= P.N) continue;
      const double val = P.off_s >= 0 ? fma(P.g, xv[c], step_scale * fma(P.d, yv[c], acc[q][c]))
                                      : fma(P.d, yv[c], fma(P.g, xv[c], acc[q][c]));
      const int64_t o = (int64_t)i * P.Out.s0 + (int64_t)j * P.Out.s1;
      if (P.Out.dtype == DT_F64) reinterpret_cast<double*>(Ob)[o] = val;
      else reinterpret_cast<float*>(Ob)[o] = (float)val;
    }
  }
}

}  // namespace

void launch_gemm64(const GemmProblem* probs, const GemmTile* tiles, int64_t ntiles, Bases b, hipStream_t s) {
  if (ntiles <= 0) return;
  hipLaunchKernelGGL(gemm64_kernel, dim3((unsigned)ntiles), dim3(256), 0, s, probs, tiles, b);
}

}  // namespace adapm
