// Split-bf16 MFMA version of the strided two-product GEMM (the "BF16X2" contraction mode):
//   Out = a1 * A1 B1 + a2 * A2 B2 + g * X + d * Y        (fp32 accumulation and output)
// used for the thin products of Alg. 2 (G R^T, L^T G, Gram matrices, factor updates) and the
// reconstruction L_{t-1}R_{t-1} - L_t R_t of eq. 3-4 on blocks with bf16 gradients.
// bf16 operands (G) are exact; an fp32 operand x travels as hi = bf16(x), lo = bf16(x - hi), and a
// product of two operands keeps hi*hi + lo*hi + hi*lo (the lo*lo term, 2^-18 relative, is dropped).
// One workgroup computes a 128 x 128 output tile; each of its four waves owns 64 x 64 (2 x 2 MFMA tiles).
// Operand tiles are staged through LDS with the contraction index contiguous, whatever the strides
// in memory (a transposed view is transposed on the way into LDS).  The next k-chunk is fetched
// into registers while the current one feeds the matrix cores.
#include "adapm_plan.h"
#include "ew_math.h"

namespace adapm {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int TM = 128, TN = 128, TK = 32;
constexpr int LS = TK + 8;                     // LDS row stride in bf16 elements (80 bytes)

union Frag {
  bf16x8 v;
  uint4 q;
};
__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  Frag f;
  f.q = *reinterpret_cast<const uint4*>(p);
  return f.v;
}

// 16 values of one 128 x 32 operand tile held by a thread between the global load and the LDS store.
struct Stage {
  float x[16];
};

// Tile element (u, k): u = row of A or column of B, k = contraction index.  Memory address of
// (u, k) is base + (u * su + k * sk) elements.
//  kfast (sk == 1): a thread takes 8 consecutive k of rows u and u + 64 (16-byte vector loads);
//  otherwise (su == 1): lanes run along u (coalesced scalar loads) and a thread takes 16 consecutive
//  k of one u, so that the transposed tile is written to LDS as whole 16-byte vectors.
__device__ __forceinline__ void fetch(const char* base, int dtype, int64_t su, int64_t sk, bool kfast, int u0, int k0,
                                      int U, int K, float alpha, Stage& st) {
  const int tid = threadIdx.x;
  if (kfast) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int gu = u0 + (tid >> 2) + 64 * h, gk = k0 + (tid & 3) * 8;
      const int64_t idx = (int64_t)gu * su + gk;
      if (gu < U && gk + 8 <= K) {
        if (dtype == DT_BF16) {
          const u32x4_a2 q = *reinterpret_cast<const u32x4_a2*>(base + idx * 2);
          const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) { st.x[8 * h + 2 * i] = __uint_as_float(w[i] << 16); st.x[8 * h + 2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
        } else {
          const f32x4_a4 a = *reinterpret_cast<const f32x4_a4*>(base + idx * 4);
          const f32x4_a4 b = *reinterpret_cast<const f32x4_a4*>(base + idx * 4 + 16);
          st.x[8 * h + 0] = a.x; st.x[8 * h + 1] = a.y; st.x[8 * h + 2] = a.z; st.x[8 * h + 3] = a.w;
          st.x[8 * h + 4] = b.x; st.x[8 * h + 5] = b.y; st.x[8 * h + 6] = b.z; st.x[8 * h + 7] = b.w;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float v = 0.f;
          if (gu < U && gk + i < K)
            v = dtype == DT_BF16 ? __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx + i]) << 16)
                                 : reinterpret_cast<const float*>(base)[idx + i];
          st.x[8 * h + i] = v;
        }
      }
    }
  } else {
    // every load is issued unconditionally on a clamped (always valid) index and masked afterwards: a
    // load inside its own bounds check would wait for the previous one, 16 latencies per chunk
    const int gu = u0 + (tid & 127), gk = k0 + 16 * (tid >> 7);
    const bool uin = gu < U;
    const int64_t jb = (int64_t)(uin ? gu : 0) * su;
    if (dtype == DT_BF16) {
      const uint16_t* src = reinterpret_cast<const uint16_t*>(base);
      uint16_t raw[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) raw[i] = src[jb + (int64_t)(gk + i < K ? gk + i : 0) * sk];
#pragma unroll
      for (int i = 0; i < 16; ++i) st.x[i] = (uin && gk + i < K) ? __uint_as_float(((uint32_t)raw[i]) << 16) : 0.f;
    } else {
      const float* src = reinterpret_cast<const float*>(base);
      float raw[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) raw[i] = src[jb + (int64_t)(gk + i < K ? gk + i : 0) * sk];
#pragma unroll
      for (int i = 0; i < 16; ++i) st.x[i] = (uin && gk + i < K) ? raw[i] : 0.f;
    }
  }
  if (alpha != 1.f) {
#pragma unroll
    for (int i = 0; i < 16; ++i) st.x[i] *= alpha;
  }
}

// registers -> LDS [u][k] as (hi, lo) bf16, 16-byte vectors in both cases
__device__ __forceinline__ void stash(const Stage& st, bool kfast, bool split, uint16_t* hi, uint16_t* lo) {
  const int tid = threadIdx.x;
  uint32_t h[8], l[8];                    // packed pairs
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (split) split_pair(st.x[2 * i], st.x[2 * i + 1], h[i], l[i]);
    else { h[i] = pack_bf16x2(st.x[2 * i], st.x[2 * i + 1]); l[i] = 0u; }
  }
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    int u, k;
    if (kfast) { u = (tid >> 2) + 64 * hh; k = (tid & 3) * 8; }
    else { u = tid & 127; k = 16 * (tid >> 7) + 8 * hh; }
    const int o = 4 * hh;
    *reinterpret_cast<uint4*>(hi + u * LS + k) = make_uint4(h[o], h[o + 1], h[o + 2], h[o + 3]);
    if (split) *reinterpret_cast<uint4*>(lo + u * LS + k) = make_uint4(l[o], l[o + 1], l[o + 2], l[o + 3]);
  }
}

// acc += alpha * A B over the whole contraction; each wave owns a 64 x 64 block = 2 x 2 MFMA tiles
__device__ __forceinline__ void product(const Mat& A, const Mat& B, float alpha, int M, int N, int K, int i0, int j0,
                                        const Bases& bs, uint16_t* Ah, uint16_t* Al, uint16_t* Bh, uint16_t* Bl,
                                        f32x16 (&acc)[2][2]) {
  const char* Ab = resolve(A.ref, bs);
  const char* Bb = resolve(B.ref, bs);
  const bool a_kfast = (A.s1 == 1), b_kfast = (B.s0 == 1);
  const bool a_split = (A.dtype != DT_BF16) || alpha != 1.f, b_split = (B.dtype != DT_BF16);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  Stage sa, sb;
  fetch(Ab, A.dtype, A.s0, A.s1, a_kfast, i0, 0, M, K, alpha, sa);
  fetch(Bb, B.dtype, B.s1, B.s0, b_kfast, j0, 0, N, K, 1.f, sb);
  for (int k0 = 0; k0 < K; k0 += TK) {
    stash(sa, a_kfast, a_split, Ah, Al);
    stash(sb, b_kfast, b_split, Bh, Bl);
    __syncthreads();
    if (k0 + TK < K) {
      fetch(Ab, A.dtype, A.s0, A.s1, a_kfast, i0, k0 + TK, M, K, alpha, sa);
      fetch(Bb, B.dtype, B.s1, B.s0, b_kfast, j0, k0 + TK, N, K, 1.f, sb);
    }
#pragma unroll
    for (int kk = 0; kk < TK / 16; ++kk) {
      const int ko = kk * 16 + 8 * lh;
      bf16x8 ah[2], bh[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        ah[t] = lds_frag(Ah + (64 * wm + 32 * t + l32) * LS + ko);
        bh[t] = lds_frag(Bh + (64 * wn + 32 * t + l32) * LS + ko);
      }
#pragma unroll
      for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[tm], bh[tn], acc[tm][tn], 0, 0, 0);
      if (a_split) {
        bf16x8 al[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) al[t] = lds_frag(Al + (64 * wm + 32 * t + l32) * LS + ko);
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
          for (int tn = 0; tn < 2; ++tn)
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[tm], bh[tn], acc[tm][tn], 0, 0, 0);
      }
      if (b_split) {
        bf16x8 bl[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) bl[t] = lds_frag(Bl + (64 * wn + 32 * t + l32) * LS + ko);
#pragma unroll
        for (int tm = 0; tm < 2; ++tm)
#pragma unroll
          for (int tn = 0; tn < 2; ++tn)
            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[tm], bl[tn], acc[tm][tn], 0, 0, 0);
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

__global__ __launch_bounds__(256, 3) void gemm_mfma_kernel(const GemmProblem* __restrict__ probs,
                                                        const GemmTile* __restrict__ tiles, Bases bs) {
  __shared__ __attribute__((aligned(16))) uint16_t Ah[TM * LS], Al[TM * LS], Bh[TN * LS], Bl[TN * LS];
  const GemmTile t = tiles[blockIdx.x];
  const GemmProblem& P = probs[t.prob];
  const int i0 = t.ti * TM, j0 = t.tj * TN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
  // the scalar factors ride on the A operand, so both products land in the same accumulators
  // a product with the gradient as an operand takes the factor of the global clipping
  if (P.K1 > 0) product(P.A1, P.B1, (float)P.a1 * (P.scale_g ? grad_scale(bs) : 1.f), P.M, P.N, P.K1, i0, j0, bs, Ah, Al, Bh, Bl, acc);
  if (P.K2 > 0) product(P.A2, P.B2, (float)P.a2, P.M, P.N, P.K2, i0, j0, bs, Ah, Al, Bh, Bl, acc);
  const char* Xb = P.X.ref.space != SP_NONE ? resolve(P.X.ref, bs) : nullptr;
  const char* Yb = P.Y.ref.space != SP_NONE ? resolve(P.Y.ref, bs) : nullptr;
  float* Ob = reinterpret_cast<float*>(resolve(P.Out.ref, bs));
  const float g = (float)P.g, d = (float)P.d;
  // optional device scalar on everything but X (normalised step of Alg. 2)
  const bool scaled = P.off_s >= 0;
  const float step_scale = scaled ? (float)*reinterpret_cast<const double*>(bs.ws + P.off_s) : 1.f;
  // X and Y are read unconditionally on clamped indices (16 independent loads at a time) and the
  // bounds check is applied to the store only
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) {
      const int j = j0 + 64 * wn + 32 * tn + l32;
      const int jc = j < P.N ? j : 0;
      float xv[16], yv[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int i = i0 + 64 * wm + 32 * tm + 8 * (e >> 2) + 4 * lh + (e & 3);
        const int ic = i < P.M ? i : 0;
        xv[e] = Xb ? load_f(Xb, P.X.dtype, (int64_t)ic * P.X.s0 + (int64_t)jc * P.X.s1) : 0.f;
        yv[e] = Yb ? load_f(Yb, P.Y.dtype, (int64_t)ic * P.Y.s0 + (int64_t)jc * P.Y.s1) : 0.f;
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int i = i0 + 64 * wm + 32 * tm + 8 * (e >> 2) + 4 * lh + (e & 3);
        if (i < P.M && j < P.N)
          Ob[(int64_t)i * P.Out.s0 + (int64_t)j * P.Out.s1] =
              scaled ? g * xv[e] + step_scale * (acc[tm][tn][e] + d * yv[e]) : acc[tm][tn][e] + g * xv[e] + d * yv[e];
      }
    }
}

}  // namespace

void launch_gemm_mfma(const GemmProblem* probs, const GemmTile* tiles, int64_t ntiles, Bases b, hipStream_t s) {
  if (ntiles <= 0) return;
  hipLaunchKernelGGL(gemm_mfma_kernel, dim3((unsigned)ntiles), dim3(256), 0, s, probs, tiles, b);
}

}  // namespace adapm
