// Fused low-rank step with R held (refresh period T > 1, steps between two runs of Alg. 2).
//
// With orthonormal rows Q = R the arg-min of Alg. 1 over L alone is a projection:
//   P   = G Q^T                                  (m x r)
//   L_t = beta1 L_{t-1} + (1-beta1) P            (least-squares fit of m_t = (1-beta1) G + beta1 L_{t-1} Q)
//   m^c = G + beta1 (L_{t-1} - P) Q              (eq. 3-4 with r_t = L_t Q - m_t)
//   W  <- W - lr (clip(m^c / (sqrt(v) + eps)) + lambda W)     (Alg. 1 last line)
// One workgroup owns a stripe of 64 rows of one block and makes two passes over it:
//   pass 1 streams G (HBM) and Q (L2) and accumulates P on the matrix cores; row sums of G^2 for
//          the blockwise second moment ride along;
//   pass 2 re-reads G (cache), reconstructs D Q tile by tile (D = beta1 (L_{t-1} - P)) and applies
//          the update to W.
// Matrix work uses v_mfma_f32_32x32x16_bf16.  G is bf16 (exact); every fp32 operand (Q, D) is
// carried as a (hi, lo) pair of bf16 values, products hi*hi + lo*hi + hi*lo accumulated in fp32
// (relative operand error 2^-17).
#include "adapm_plan.h"

namespace adapm {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 64;     // rows per stripe
constexpr int BK = 64;     // columns per chunk of pass 1
constexpr int BN = 64;     // columns per chunk of pass 2
constexpr int GS = BK + 8; // LDS row strides (elements), padded so 16-byte fragment reads spread over all banks
constexpr int CS = BN + 8;

__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// x -> (hi, lo) with hi = bf16(x), lo = bf16(x - hi)
__device__ __forceinline__ void split2(float x, uint32_t& hi, uint32_t& lo) {
  hi = bf16_rne_bits(x);
  lo = bf16_rne_bits(x - __uint_as_float(hi << 16));
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

union Frag {
  bf16x8 v;
  uint4 q;
};

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  Frag f;
  f.q = *reinterpret_cast<const uint4*>(p);
  return f.v;
}

__device__ __forceinline__ float update_elem(float w, float mc, float v, const StepScalars& sc, float lrs, float wd) {
  float u = (mc * sc.inv_debias_m) / (sqrtf(v * sc.inv_debias_v) + sc.eps);
  u = fminf(fmaxf(u, -sc.clip), sc.clip);
  return w - lrs * (u + wd * w);
}

template <int RT>
__global__ __launch_bounds__(256, 2) void proj_kernel(const ProjItem* __restrict__ items,
                                                      const LrBlockDev* __restrict__ lrb, Bases bs, StepScalars sc) {
  constexpr int R = 32 * RT;
  constexpr int DS = R + 8;                         // LDS row stride of the r-contiguous arrays
  constexpr int TPW = (2 * RT >= 4) ? (2 * RT / 4) : 1;   // pass-1 output tiles per wave
  constexpr int P1_BYTES = (BM * GS + 2 * R * GS) * 2;
  constexpr int P2_BYTES = 2 * BN * DS * 2 + BM * CS * 4;
  constexpr int D_BYTES = 2 * BM * DS * 2;
  constexpr int SMEM = (P1_BYTES > P2_BYTES ? (P1_BYTES > D_BYTES ? P1_BYTES : D_BYTES)
                                            : (P2_BYTES > D_BYTES ? P2_BYTES : D_BYTES));
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ float vrow[BM];
  __shared__ float rsum[BM];

  const ProjItem item = items[blockIdx.x];
  if (item.lr < 0) return;
  const LrBlockDev B = lrb[item.lr];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int m = B.m, n = B.n, row0 = item.row0;
  const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(bs.grads[B.block]);
  char* __restrict__ W = reinterpret_cast<char*>(bs.params[B.block]);
  float* __restrict__ Lst = reinterpret_cast<float*>(bs.state + B.off_L);
  const float* __restrict__ Q = reinterpret_cast<const float*>(bs.state + B.off_Q);
  float* __restrict__ vst = reinterpret_cast<float*>(bs.state + B.off_v);
  const uint16_t* __restrict__ Qth_g = reinterpret_cast<const uint16_t*>(bs.ws + B.off_Qt_hi);
  const uint16_t* __restrict__ Qtl_g = reinterpret_cast<const uint16_t*>(bs.ws + B.off_Qt_lo);

  // ------------------------------------------------------------------ pass 1: P = G Q^T
  uint16_t* Gs = reinterpret_cast<uint16_t*>(smem);               // [BM][GS]
  uint16_t* Qh = Gs + BM * GS;                                    // [R][GS]
  uint16_t* Ql = Qh + R * GS;                                     // [R][GS]
  f32x16 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
  float ss0 = 0.f, ss1 = 0.f;                                      // sums of g^2: rows tid/8 and 32 + tid/8
  const bool p1_active = wave < 2 * RT;                           // r = 32: only two output tiles
  const int my_nt = (RT >= 4) ? wave : (wave % RT);
  const int my_mt0 = (RT >= 4) ? 0 : (wave / RT);

  for (int k0 = 0; k0 < n; k0 += BK) {
    // stage G chunk (bf16, 16-byte vectors) and accumulate the row sums of squares
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      uint4 q = make_uint4(0, 0, 0, 0);
      if (row0 + row < m && k0 + c8 < n) q = *reinterpret_cast<const uint4*>(G + (int64_t)(row0 + row) * n + k0 + c8);
      *reinterpret_cast<uint4*>(Gs + row * GS + c8) = q;
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) { const float a = bf16_lo(w[j]), b = bf16_hi(w[j]); s += a * a + b * b; }
      if (i == 0) ss0 += s; else ss1 += s;
    }
    // stage Q chunk: fp32 -> (hi, lo) bf16
#pragma unroll
    for (int i = 0; i < (R * BK / 4) / 256; ++i) {
      const int id = tid + 256 * i, a = id >> 4, c4 = (id & 15) * 4;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k0 + c4 < n) x = *reinterpret_cast<const float4*>(Q + (int64_t)a * n + k0 + c4);
      uint32_t h0, l0, h1, l1, h2, l2, h3, l3;
      split2(x.x, h0, l0); split2(x.y, h1, l1); split2(x.z, h2, l2); split2(x.w, h3, l3);
      *reinterpret_cast<uint2*>(Qh + a * GS + c4) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
      *reinterpret_cast<uint2*>(Ql + a * GS + c4) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
    }
    __syncthreads();
    if (p1_active) {
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int ko = kk * 16 + 8 * lh;
        const bf16x8 bh = lds_frag(Qh + (32 * my_nt + l32) * GS + ko);
        const bf16x8 bl = lds_frag(Ql + (32 * my_nt + l32) * GS + ko);
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
          const bf16x8 a = lds_frag(Gs + (32 * (my_mt0 + t) + l32) * GS + ko);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl, acc[t], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // ------------------------------------------------------------------ second moment of the stripe
  // a row is covered by 8 consecutive lanes
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) { ss0 += __shfl_xor(ss0, o, 64); ss1 += __shfl_xor(ss1, o, 64); }
  if ((tid & 7) == 0) { rsum[tid >> 3] = ss0; rsum[32 + (tid >> 3)] = ss1; }
  __syncthreads();
  if (B.v_kind == 1) {             // groups of v_group_rows rows inside the stripe: finish v here
    const int g = B.v_group_rows;
    if (tid < BM / g) {
      const int r0 = tid * g;
      if (row0 + r0 < m) {
        double s = 0.0;
        for (int i = 0; i < g; ++i) s += (double)rsum[r0 + i];
        float* vp = vst + (row0 + r0) / g;
        const float vn = (float)((double)sc.beta2 * (double)*vp + (1.0 - (double)sc.beta2) * (s / ((double)g * (double)n)));
        *vp = vn;
        for (int i = 0; i < g; ++i) vrow[r0 + i] = vn;
      }
    }
  } else if (B.v_kind == 2) {      // v finished by the statistics kernel: one value per group of rows
    if (tid < BM && row0 + tid < m) vrow[tid] = vst[(row0 + tid) / B.v_group_rows];
  }

  // ------------------------------------------------------------------ L_t and D = dL L' + dP P
  uint16_t* Dh = reinterpret_cast<uint16_t*>(smem);               // [BM][DS]
  uint16_t* Dl = Dh + BM * DS;
  if (p1_active) {
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const int col = 32 * my_nt + l32;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = 32 * (my_mt0 + t) + 8 * q + 4 * lh + p;
          float d = 0.f;
          if (row0 + row < m) {
            float* lp = Lst + (int64_t)(row0 + row) * R + col;
            const float lprev = *lp, pv = acc[t][4 * q + p];
            *lp = sc.beta1 * lprev + (1.f - sc.beta1) * pv;
            d = sc.dL * lprev + sc.dP * pv;
          }
          uint32_t h, l;
          split2(d, h, l);
          Dh[row * DS + col] = (uint16_t)h;
          Dl[row * DS + col] = (uint16_t)l;
        }
    }
  }
  __syncthreads();
  // A fragments of D for this wave's 32 rows stay in registers for the whole of pass 2
  const int wr = wave & 1, wc = wave >> 1;
  bf16x8 dh[2 * RT], dl[2 * RT];
#pragma unroll
  for (int ks = 0; ks < 2 * RT; ++ks) {
    dh[ks] = lds_frag(Dh + (32 * wr + l32) * DS + 16 * ks + 8 * lh);
    dl[ks] = lds_frag(Dl + (32 * wr + l32) * DS + 16 * ks + 8 * lh);
  }
  __syncthreads();

  // ------------------------------------------------------------------ pass 2: C = D Q, update W
  uint16_t* Th = reinterpret_cast<uint16_t*>(smem);               // [BN][DS]  Q^T hi
  uint16_t* Tl = Th + BN * DS;                                    // [BN][DS]  Q^T lo
  float* Cs = reinterpret_cast<float*>(smem + 2 * BN * DS * 2);   // [BM][CS]
  const float lrs = sc.lr * B.lr_scale, wd = B.wd;
  const float ob2 = 1.f - sc.beta2;
  for (int j0 = 0; j0 < n; j0 += BN) {
#pragma unroll
    for (int i = 0; i < (BN * R / 8) / 256; ++i) {
      const int id = tid + 256 * i, j = id / (R / 8), a8 = (id % (R / 8)) * 8;
      uint4 h = make_uint4(0, 0, 0, 0), l = make_uint4(0, 0, 0, 0);
      if (j0 + j < n) {
        h = *reinterpret_cast<const uint4*>(Qth_g + (int64_t)(j0 + j) * R + a8);
        l = *reinterpret_cast<const uint4*>(Qtl_g + (int64_t)(j0 + j) * R + a8);
      }
      *reinterpret_cast<uint4*>(Th + j * DS + a8) = h;
      *reinterpret_cast<uint4*>(Tl + j * DS + a8) = l;
    }
    __syncthreads();
    f32x16 c;
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) {
      const bf16x8 bh = lds_frag(Th + (32 * wc + l32) * DS + 16 * ks + 8 * lh);
      const bf16x8 bl = lds_frag(Tl + (32 * wc + l32) * DS + 16 * ks + 8 * lh);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bh, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks], bh, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bl, c, 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int p = 0; p < 4; ++p) Cs[(32 * wr + 8 * q + 4 * lh + p) * CS + 32 * wc + l32] = c[4 * q + p];
    __syncthreads();
    // element-wise tail on 8 consecutive columns per thread
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      if (row0 + row >= m || j0 + c8 >= n) continue;
      const int64_t e = (int64_t)(row0 + row) * n + j0 + c8;
      const uint4 gq = *reinterpret_cast<const uint4*>(G + e);
      const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
      float g[8], w[8], mc[8], vv[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) { g[2 * j] = bf16_lo(gw[j]); g[2 * j + 1] = bf16_hi(gw[j]); }
      const float4 ca = *reinterpret_cast<const float4*>(Cs + row * CS + c8);
      const float4 cb = *reinterpret_cast<const float4*>(Cs + row * CS + c8 + 4);
      const float cc[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) mc[j] = sc.cG * g[j] + sc.cC * cc[j];
      if (B.v_kind == 0) {          // per-element second moment
        float4* vp = reinterpret_cast<float4*>(vst + e);
        float4 va = vp[0], vb = vp[1];
        vv[0] = va.x; vv[1] = va.y; vv[2] = va.z; vv[3] = va.w; vv[4] = vb.x; vv[5] = vb.y; vv[6] = vb.z; vv[7] = vb.w;
#pragma unroll
        for (int j = 0; j < 8; ++j) vv[j] = sc.beta2 * vv[j] + ob2 * g[j] * g[j];
        vp[0] = make_float4(vv[0], vv[1], vv[2], vv[3]);
        vp[1] = make_float4(vv[4], vv[5], vv[6], vv[7]);
      } else {
        const float x = vrow[row];
#pragma unroll
        for (int j = 0; j < 8; ++j) vv[j] = x;
      }
      if (B.param_dtype == DT_BF16) {
        uint4* wp = reinterpret_cast<uint4*>(W + e * 2);
        const uint4 wq = *wp;
        const uint32_t ww[4] = {wq.x, wq.y, wq.z, wq.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) { w[2 * j] = bf16_lo(ww[j]); w[2 * j + 1] = bf16_hi(ww[j]); }
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float a = update_elem(w[2 * j], mc[2 * j], vv[2 * j], sc, lrs, wd);
          const float b = update_elem(w[2 * j + 1], mc[2 * j + 1], vv[2 * j + 1], sc, lrs, wd);
          o[j] = bf16_rne_bits(a) | (bf16_rne_bits(b) << 16);
        }
        *wp = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
        float4* wp = reinterpret_cast<float4*>(W + e * 4);
        const float4 wa = wp[0], wb = wp[1];
        w[0] = wa.x; w[1] = wa.y; w[2] = wa.z; w[3] = wa.w; w[4] = wb.x; w[5] = wb.y; w[6] = wb.z; w[7] = wb.w;
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = update_elem(w[j], mc[j], vv[j], sc, lrs, wd);
        wp[0] = make_float4(w[0], w[1], w[2], w[3]);
        wp[1] = make_float4(w[4], w[5], w[6], w[7]);
      }
    }
  }
}

// Q (r x n fp32, state) -> Q^T as bf16 (hi, lo) pairs, [n][r], in the workspace.
__global__ __launch_bounds__(256) void qsplit_kernel(const QsItem* __restrict__ items,
                                                     const LrBlockDev* __restrict__ lrb, Bases bs) {
  __shared__ float tile[32][65];
  const QsItem it = items[blockIdx.x];
  const LrBlockDev B = lrb[it.lr];
  const int n = B.n, R = B.r;
  const float* __restrict__ Q = reinterpret_cast<const float*>(bs.state + B.off_Q);
  uint16_t* __restrict__ Th = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qt_hi);
  uint16_t* __restrict__ Tl = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qt_lo);
  const int a0 = it.a0, j0 = it.j0, tid = threadIdx.x;
  // read 32 rows (a) x 64 columns (j), j fastest
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = tid + 256 * i, a = id >> 6, j = id & 63;
    tile[a][j] = (a0 + a < R && j0 + j < n) ? Q[(int64_t)(a0 + a) * n + j0 + j] : 0.f;
  }
  __syncthreads();
  // write 64 rows (j) x 32 columns (a), a fastest
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = tid + 256 * i, j = id >> 5, a = id & 31;
    if (a0 + a < R && j0 + j < n) {
      uint32_t h, l;
      split2(tile[a][j], h, l);
      Th[(int64_t)(j0 + j) * R + a0 + a] = (uint16_t)h;
      Tl[(int64_t)(j0 + j) * R + a0 + a] = (uint16_t)l;
    }
  }
}

}  // namespace

void launch_proj(int rt, const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, StepScalars sc,
                 hipStream_t s) {
  if (nitems <= 0) return;
  const dim3 grid((unsigned)nitems), block(256);
  if (rt == 1) hipLaunchKernelGGL(proj_kernel<1>, grid, block, 0, s, items, lrb, b, sc);
  else if (rt == 2) hipLaunchKernelGGL(proj_kernel<2>, grid, block, 0, s, items, lrb, b, sc);
  else hipLaunchKernelGGL(proj_kernel<4>, grid, block, 0, s, items, lrb, b, sc);
}

void launch_qsplit(const QsItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(qsplit_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, lrb, b);
}

}  // namespace adapm
