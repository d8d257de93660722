// Split-bf16 MFMA version of the strided two-product GEMM (the "BF16X2" contraction mode):
//   Out = a1 * A1 B1 + a2 * A2 B2 + g * X + d * Y        (fp32 accumulation and output)
// used for the thin products of Alg. 2 (G R^T, L^T G, Gram matrices, factor updates) and the
// reconstruction L_{t-1}R_{t-1} - L_t R_t of eq. 3-4 on blocks with bf16 gradients.
// bf16 operands (G) are exact; an fp32 operand x travels as hi = bf16(x), lo = bf16(x - hi), and a
// product of two operands keeps hi*hi + lo*hi + hi*lo (the lo*lo term, 2^-18 relative, is dropped).
// One workgroup computes a 64 x 64 output tile; each of its four waves owns a 32 x 32 MFMA tile.
// Operand tiles are staged through LDS with the contraction index contiguous, whatever the strides
// in memory (a transposed view is transposed on the way into LDS).  The next k-chunk is fetched
// into registers while the current one feeds the matrix cores.
#include "adapm_plan.h"

namespace adapm {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int TM = 64, TN = 64, TK = 32;
constexpr int LS = TK + 8;                     // LDS row stride in bf16 elements (80 bytes)

__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

union Frag {
  bf16x8 v;
  uint4 q;
};
__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  Frag f;
  f.q = *reinterpret_cast<const uint4*>(p);
  return f.v;
}

// 8 values of one operand tile held by a thread between the global load and the LDS store.
struct Stage {
  float x[8];
};

// Tile element (u, k): u = row of A or column of B, k = contraction index.  Memory address of
// (u, k) is base + (u * su + k * sk) elements.  kfast (sk == 1): a thread takes 8 consecutive k of
// one u; otherwise (su == 1) it takes 8 consecutive u of one k.
__device__ __forceinline__ void fetch(const char* base, int dtype, int64_t su, int64_t sk, bool kfast, int u0, int k0,
                                      int U, int K, Stage& st) {
  const int tid = threadIdx.x;
  int u, k, du, dk;
  if (kfast) { u = tid >> 2; k = (tid & 3) * 8; du = 0; dk = 1; }
  else { k = tid >> 3; u = (tid & 7) * 8; du = 1; dk = 0; }
  const int gu = u0 + u, gk = k0 + k;
  const int64_t idx = (int64_t)gu * su + (int64_t)gk * sk;
  const bool full = kfast ? (gu < U && gk + 8 <= K) : (gk < K && gu + 8 <= U);
  if (full) {
    if (dtype == DT_BF16) {
      const uint4 q = *reinterpret_cast<const uint4*>(base + idx * 2);
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) { st.x[2 * i] = __uint_as_float(w[i] << 16); st.x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    } else {
      const float4 a = *reinterpret_cast<const float4*>(base + idx * 4);
      const float4 b = *reinterpret_cast<const float4*>(base + idx * 4 + 16);
      st.x[0] = a.x; st.x[1] = a.y; st.x[2] = a.z; st.x[3] = a.w; st.x[4] = b.x; st.x[5] = b.y; st.x[6] = b.z; st.x[7] = b.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int eu = gu + i * du, ek = gk + i * dk;
      float v = 0.f;
      if (eu < U && ek < K) {
        const int64_t j = (int64_t)eu * su + (int64_t)ek * sk;
        v = dtype == DT_BF16 ? __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(base)[j]) << 16)
                             : reinterpret_cast<const float*>(base)[j];
      }
      st.x[i] = v;
    }
  }
}

// registers -> LDS [u][k] as (hi, lo) bf16
__device__ __forceinline__ void stash(const Stage& st, bool kfast, bool split, uint16_t* hi, uint16_t* lo) {
  const int tid = threadIdx.x;
  uint32_t h[8], l[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    h[i] = bf16_rne_bits(st.x[i]);
    l[i] = split ? bf16_rne_bits(st.x[i] - __uint_as_float(h[i] << 16)) : 0u;
  }
  if (kfast) {
    const int u = tid >> 2, k = (tid & 3) * 8;
    *reinterpret_cast<uint4*>(hi + u * LS + k) = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    if (split)
      *reinterpret_cast<uint4*>(lo + u * LS + k) = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
  } else {
    const int k = tid >> 3, u = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      hi[(u + i) * LS + k] = (uint16_t)h[i];
      if (split) lo[(u + i) * LS + k] = (uint16_t)l[i];
    }
  }
}

__device__ __forceinline__ void product(const Mat& A, const Mat& B, int M, int N, int K, int i0, int j0, const Bases& bs,
                                        uint16_t* Ah, uint16_t* Al, uint16_t* Bh, uint16_t* Bl, f32x16& acc) {
  const char* Ab = resolve(A.ref, bs);
  const char* Bb = resolve(B.ref, bs);
  const bool a_kfast = (A.s1 == 1), b_kfast = (B.s0 == 1);
  const bool a_split = (A.dtype != DT_BF16), b_split = (B.dtype != DT_BF16);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  Stage sa, sb;
  fetch(Ab, A.dtype, A.s0, A.s1, a_kfast, i0, 0, M, K, sa);
  fetch(Bb, B.dtype, B.s1, B.s0, b_kfast, j0, 0, N, K, sb);
  for (int k0 = 0; k0 < K; k0 += TK) {
    stash(sa, a_kfast, a_split, Ah, Al);
    stash(sb, b_kfast, b_split, Bh, Bl);
    __syncthreads();
    if (k0 + TK < K) {
      fetch(Ab, A.dtype, A.s0, A.s1, a_kfast, i0, k0 + TK, M, K, sa);
      fetch(Bb, B.dtype, B.s1, B.s0, b_kfast, j0, k0 + TK, N, K, sb);
    }
#pragma unroll
    for (int kk = 0; kk < TK / 16; ++kk) {
      const int ko = kk * 16 + 8 * lh;
      const bf16x8 ah = lds_frag(Ah + (32 * wm + l32) * LS + ko);
      const bf16x8 bh = lds_frag(Bh + (32 * wn + l32) * LS + ko);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
      if (a_split) {
        const bf16x8 al = lds_frag(Al + (32 * wm + l32) * LS + ko);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
      }
      if (b_split) {
        const bf16x8 bl = lds_frag(Bl + (32 * wn + l32) * LS + ko);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
      }
    }
    __syncthreads();
  }
}

__device__ __forceinline__ float load_f(const char* base, int dtype, int64_t idx) {
  if (dtype == DT_F32) return reinterpret_cast<const float*>(base)[idx];
  if (dtype == DT_BF16) return __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx]) << 16);
  return (float)reinterpret_cast<const double*>(base)[idx];
}

__global__ __launch_bounds__(256) void gemm_mfma_kernel(const GemmProblem* __restrict__ probs,
                                                        const GemmTile* __restrict__ tiles, Bases bs) {
  __shared__ __attribute__((aligned(16))) uint16_t Ah[TM * LS], Al[TM * LS], Bh[TN * LS], Bl[TN * LS];
  const GemmTile t = tiles[blockIdx.x];
  const GemmProblem& P = probs[t.prob];
  const int i0 = t.ti * TM, j0 = t.tj * TN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  if (P.K1 > 0) {
    product(P.A1, P.B1, P.M, P.N, P.K1, i0, j0, bs, Ah, Al, Bh, Bl, acc);
    const float a1 = (float)P.a1;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] *= a1;
  }
  if (P.K2 > 0) {
    f32x16 acc2;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc2[i] = 0.f;
    product(P.A2, P.B2, P.M, P.N, P.K2, i0, j0, bs, Ah, Al, Bh, Bl, acc2);
    const float a2 = (float)P.a2;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] += a2 * acc2[i];
  }
  const char* Xb = P.X.ref.space != SP_NONE ? resolve(P.X.ref, bs) : nullptr;
  const char* Yb = P.Y.ref.space != SP_NONE ? resolve(P.Y.ref, bs) : nullptr;
  float* Ob = reinterpret_cast<float*>(resolve(P.Out.ref, bs));
  const float g = (float)P.g, d = (float)P.d;
  const int j = j0 + 32 * wn + l32;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int i = i0 + 32 * wm + 8 * q + 4 * lh + p;
      if (i < P.M && j < P.N) {
        float val = acc[4 * q + p];
        if (Xb) val += g * load_f(Xb, P.X.dtype, (int64_t)i * P.X.s0 + (int64_t)j * P.X.s1);
        if (Yb) val += d * load_f(Yb, P.Y.dtype, (int64_t)i * P.Y.s0 + (int64_t)j * P.Y.s1);
        Ob[(int64_t)i * P.Out.s0 + (int64_t)j * P.Out.s1] = val;
      }
    }
}

}  // namespace

void launch_gemm_mfma(const GemmProblem* probs, const GemmTile* tiles, int64_t ntiles, Bases b, hipStream_t s) {
  if (ntiles <= 0) return;
  hipLaunchKernelGGL(gemm_mfma_kernel, dim3((unsigned)ntiles), dim3(256), 0, s, probs, tiles, b);
}

}  // namespace adapm
