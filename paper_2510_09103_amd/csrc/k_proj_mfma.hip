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
#include "ew_math.h"

namespace adapm {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 64;     // rows per stripe
constexpr int BK = 64;     // columns per chunk of pass 1
constexpr int BN = 64;     // columns per chunk of pass 2
constexpr int GS = BK + 8; // LDS row strides (elements), padded so 16-byte fragment reads spread over all banks
constexpr int CS = BN + 8;

union Frag {
  bf16x8 v;
  uint4 q;
};

__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) {
  Frag f;
  f.q = *reinterpret_cast<const uint4*>(p);
  return f.v;
}

template <int RT>
__global__ __launch_bounds__(256, 2) void proj_kernel(const ProjItem* __restrict__ items,
                                                      const LrBlockDev* __restrict__ lrb, Bases bs, StepScalars sc) {
  constexpr int R = 32 * RT;
  constexpr int DS = R + 8;                         // LDS row stride of the r-contiguous arrays
  constexpr int TPW = (2 * RT >= 4) ? (2 * RT / 4) : 1;   // pass-1 output tiles per wave
  constexpr int P1_BYTES = (BM * GS + 2 * R * GS) * 2;
  constexpr int P2_BYTES = 2 * BN * DS * 2 + BM * CS * 4;
  constexpr int D_BYTES = (2 * BM * DS * 2 > BM * (R + 4) * 4) ? 2 * BM * DS * 2 : BM * (R + 4) * 4;
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
  const uint16_t* __restrict__ Qnh_g = reinterpret_cast<const uint16_t*>(bs.ws + B.off_Qn_hi);
  const uint16_t* __restrict__ Qnl_g = reinterpret_cast<const uint16_t*>(bs.ws + B.off_Qn_lo);

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

  // The next chunk travels from memory into registers while the matrix cores work on the
  // current one (one memory round trip per chunk would otherwise be exposed at every barrier).
  constexpr int QV = (R * BK / 8) / 256;                           // 16-byte loads of Q per thread, chunk and half
  uint4 ga[2], gb[2];                                              // G: two chunks ahead (bytes in flight)
  uint4 qhp[QV], qlp[QV];                                          // Q (hi, lo): one chunk ahead (comes from L2)
  auto fetch_g = [&](int k0, uint4 (&dst)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      dst[i] = make_uint4(0, 0, 0, 0);
      if (row0 + row < m && k0 + c8 < n && !(sc.dbg & 128))
        dst[i] = *reinterpret_cast<const uint4*>(G + (int64_t)(row0 + row) * n + k0 + c8);
    }
  };
  auto fetch_q = [&](int k0) {
#pragma unroll
    for (int i = 0; i < QV; ++i) {
      const int id = tid + 256 * i, a = id >> 3, c8 = (id & 7) * 8;
      qhp[i] = make_uint4(0, 0, 0, 0);
      qlp[i] = make_uint4(0, 0, 0, 0);
      if (k0 + c8 < n && !(sc.dbg & 2)) {
        qhp[i] = *reinterpret_cast<const uint4*>(Qnh_g + (int64_t)a * n + k0 + c8);
        qlp[i] = *reinterpret_cast<const uint4*>(Qnl_g + (int64_t)a * n + k0 + c8);
      }
    }
  };
  // one chunk: registers -> LDS, refill the registers, matrix cores on the LDS copy
  auto chunk = [&](int k0, uint4 (&gcur)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      const uint4 q = gcur[i];
      *reinterpret_cast<uint4*>(Gs + row * GS + c8) = q;
      const float s = dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
      if (i == 0) ss0 += s; else ss1 += s;
    }
#pragma unroll
    for (int i = 0; i < QV; ++i) {
      const int id = tid + 256 * i, a = id >> 3, c8 = (id & 7) * 8;
      *reinterpret_cast<uint4*>(Qh + a * GS + c8) = qhp[i];
      *reinterpret_cast<uint4*>(Ql + a * GS + c8) = qlp[i];
    }
    __syncthreads();
    if (k0 + 2 * BK < n) fetch_g(k0 + 2 * BK, gcur);
    if (k0 + BK < n) fetch_q(k0 + BK);
    if (p1_active && !(sc.dbg & 1)) {
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
  };
  fetch_g(0, ga);
  fetch_g(BK, gb);
  fetch_q(0);
  for (int k0 = 0; k0 < ((sc.dbg & 1024) ? 0 : n); k0 += 2 * BK) {
    chunk(k0, ga);
    if (k0 + BK < n) chunk(k0 + BK, gb);
  }

  // ------------------------------------------------------------------ second moment of the stripe
  // a row is covered by 8 consecutive lanes
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) { ss0 += __shfl_xor(ss0, o, 64); ss1 += __shfl_xor(ss1, o, 64); }
  if ((tid & 7) == 0) { rsum[tid >> 3] = ss0; rsum[32 + (tid >> 3)] = ss1; }
  __syncthreads();
  if (sc.dbg & 512) {} else if (B.v_kind == 1) {             // groups of v_group_rows rows inside the stripe: finish v here
    const int g = B.v_group_rows;
    if (tid < BM / g) {
      const int r0 = tid * g;
      if (row0 + r0 < m) {
        double s = 0.0;
        for (int i = 0; i < g; ++i) s += (double)rsum[r0 + i];
        float* vp = vst + (row0 + r0) / g;
        const float vn = (float)((double)sc.beta2 * (double)*vp + (1.0 - (double)sc.beta2) * (s / ((double)g * (double)n)));
        *vp = vn;
        const float inv = inv_denom_exact(vn, sc.inv_debias_v, sc.inv_debias_m, sc.eps);
        for (int i = 0; i < g; ++i) vrow[r0 + i] = inv;
      }
    }
  } else if (B.v_kind == 2) {      // v finished by the statistics kernel: one value per group of rows
    if (tid < BM && row0 + tid < m)
      vrow[tid] = inv_denom_exact(vst[(row0 + tid) / B.v_group_rows], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
  }

  // ------------------------------------------------------------------ L_t and D = dL L' + dP P
  // P leaves the accumulators through LDS so that L is read and written as whole rows (float4).
  float* Ps = reinterpret_cast<float*>(smem);                     // [BM][R + 4] fp32
  constexpr int PS = R + 4;
  if (p1_active && !(sc.dbg & 256)) {
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const int col = 32 * my_nt + l32;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = 0; p < 4; ++p) Ps[(32 * (my_mt0 + t) + 8 * q + 4 * lh + p) * PS + col] = acc[t][4 * q + p];
    }
  }
  __syncthreads();
  constexpr int LV = (BM * R / 4) / 256;                          // float4 per thread
  uint2 dhv[LV], dlv[LV];
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int id = tid + 256 * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
    float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row0 + row < m && !(sc.dbg & 256)) {
      float4* lp = reinterpret_cast<float4*>(Lst + (int64_t)(row0 + row) * R + c4);
      const float4 lprev = *lp;
      const float4 pv = *reinterpret_cast<const float4*>(Ps + row * PS + c4);
      const float b1 = sc.beta1, ob1 = 1.f - sc.beta1;
      *lp = make_float4(b1 * lprev.x + ob1 * pv.x, b1 * lprev.y + ob1 * pv.y, b1 * lprev.z + ob1 * pv.z,
                        b1 * lprev.w + ob1 * pv.w);
      d = make_float4(sc.dL * lprev.x + sc.dP * pv.x, sc.dL * lprev.y + sc.dP * pv.y, sc.dL * lprev.z + sc.dP * pv.z,
                      sc.dL * lprev.w + sc.dP * pv.w);
    }
    uint32_t h0, l0, h1, l1;
    split_pair(d.x, d.y, h0, l0);
    split_pair(d.z, d.w, h1, l1);
    dhv[i] = make_uint2(h0, h1);
    dlv[i] = make_uint2(l0, l1);
  }
  __syncthreads();                                                 // Ps is dead, D takes its place
  uint16_t* Dh = reinterpret_cast<uint16_t*>(smem);               // [BM][DS]
  uint16_t* Dl = Dh + BM * DS;
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int id = tid + 256 * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
    *reinterpret_cast<uint2*>(Dh + row * DS + c4) = dhv[i];
    *reinterpret_cast<uint2*>(Dl + row * DS + c4) = dlv[i];
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
  const UpdCoef cf = make_coef(sc.lr, B.lr_scale, B.wd, sc.clip);
  const float ob2 = 1.f - sc.beta2;
  constexpr int TV = (BN * R / 8) / 256;                          // 16-byte loads of Q^T per thread, chunk and half
  uint4 thp[TV], tlp[TV];                                          // next chunk of Q^T (hi, lo)
  uint4 gcur[2], wcur[4], gnxt[2], wnxt[4];                        // G / W vectors of this and the next chunk
  const bool w16 = B.param_dtype == DT_BF16;
  auto fetch_t = [&](int j0) {
#pragma unroll
    for (int i = 0; i < TV; ++i) {
      const int id = tid + 256 * i, j = id / (R / 8), a8 = (id % (R / 8)) * 8;
      thp[i] = make_uint4(0, 0, 0, 0);
      tlp[i] = make_uint4(0, 0, 0, 0);
      if (j0 + j < n && !(sc.dbg & 8)) {
        thp[i] = *reinterpret_cast<const uint4*>(Qth_g + (int64_t)(j0 + j) * R + a8);
        tlp[i] = *reinterpret_cast<const uint4*>(Qtl_g + (int64_t)(j0 + j) * R + a8);
      }
    }
  };
  auto fetch_gw = [&](int j0, uint4* gq, uint4* wq) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      gq[i] = make_uint4(0, 0, 0, 0);
      wq[2 * i] = wq[2 * i + 1] = make_uint4(0, 0, 0, 0);
      if (row0 + row < m && j0 + c8 < n && !(sc.dbg & 16)) {
        const int64_t e = (int64_t)(row0 + row) * n + j0 + c8;
        gq[i] = *reinterpret_cast<const uint4*>(G + e);
        if (w16) {
          wq[2 * i] = *reinterpret_cast<const uint4*>(W + e * 2);
        } else {
          wq[2 * i] = *reinterpret_cast<const uint4*>(W + e * 4);
          wq[2 * i + 1] = *reinterpret_cast<const uint4*>(W + e * 4 + 16);
        }
      }
    }
  };
  fetch_t(0);
  fetch_gw(0, gcur, wcur);
  for (int j0 = 0; j0 < ((sc.dbg & 64) ? 0 : n); j0 += BN) {
#pragma unroll
    for (int i = 0; i < TV; ++i) {
      const int id = tid + 256 * i, j = id / (R / 8), a8 = (id % (R / 8)) * 8;
      *reinterpret_cast<uint4*>(Th + j * DS + a8) = thp[i];
      *reinterpret_cast<uint4*>(Tl + j * DS + a8) = tlp[i];
    }
    __syncthreads();
    if (j0 + BN < n) {
      fetch_t(j0 + BN);
      fetch_gw(j0 + BN, gnxt, wnxt);
    }
    f32x16 c;
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = 0.f;
if (!(sc.dbg & 4))
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
      if (row0 + row >= m || j0 + c8 >= n || (sc.dbg & 32)) continue;
      const int64_t e = (int64_t)(row0 + row) * n + j0 + c8;
      const uint32_t gw[4] = {gcur[i].x, gcur[i].y, gcur[i].z, gcur[i].w};
      float g[8], mc[8], inv[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) { g[2 * j] = bf16lo(gw[j]); g[2 * j + 1] = bf16hi(gw[j]); }
      const float4 ca = *reinterpret_cast<const float4*>(Cs + row * CS + c8);
      const float4 cb = *reinterpret_cast<const float4*>(Cs + row * CS + c8 + 4);
      const float cc[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
#pragma unroll
      for (int j = 0; j < 8; ++j) mc[j] = fmaf(sc.cC, cc[j], sc.cG * g[j]);
      if (B.v_kind == 0) {          // per-element second moment
        float4* vp = reinterpret_cast<float4*>(vst + e);
        const float4 va = vp[0], vb = vp[1];
        float vv[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          vv[j] = sc.beta2 * vv[j] + ob2 * g[j] * g[j];
          inv[j] = inv_denom_fast(vv[j], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
        }
        vp[0] = make_float4(vv[0], vv[1], vv[2], vv[3]);
        vp[1] = make_float4(vv[4], vv[5], vv[6], vv[7]);
      } else {
        const float x = vrow[row];
#pragma unroll
        for (int j = 0; j < 8; ++j) inv[j] = x;
      }
      if (w16) {
        const uint32_t ww[4] = {wcur[2 * i].x, wcur[2 * i].y, wcur[2 * i].z, wcur[2 * i].w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          o[j] = pack_bf16x2(apply_update(bf16lo(ww[j]), mc[2 * j], inv[2 * j], cf),
                             apply_update(bf16hi(ww[j]), mc[2 * j + 1], inv[2 * j + 1], cf));
        *reinterpret_cast<uint4*>(W + e * 2) = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
        const uint32_t ww[8] = {wcur[2 * i].x, wcur[2 * i].y, wcur[2 * i].z, wcur[2 * i].w,
                                wcur[2 * i + 1].x, wcur[2 * i + 1].y, wcur[2 * i + 1].z, wcur[2 * i + 1].w};
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = apply_update(__uint_as_float(ww[j]), mc[j], inv[j], cf);
        float4* wp = reinterpret_cast<float4*>(W + e * 4);
        wp[0] = make_float4(w[0], w[1], w[2], w[3]);
        wp[1] = make_float4(w[4], w[5], w[6], w[7]);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) { gcur[i] = gnxt[i]; wcur[2 * i] = wnxt[2 * i]; wcur[2 * i + 1] = wnxt[2 * i + 1]; }
  }
}

// Q (r x n fp32, state) -> bf16 (hi, lo) pairs in the workspace, both as Q [r][n] and as Q^T [n][r].
__global__ __launch_bounds__(256) void qsplit_kernel(const QsItem* __restrict__ items,
                                                     const LrBlockDev* __restrict__ lrb, Bases bs) {
  __shared__ float tile[32][65];
  const QsItem it = items[blockIdx.x];
  const LrBlockDev B = lrb[it.lr];
  const int n = B.n, R = B.r;
  const float* __restrict__ Q = reinterpret_cast<const float*>(bs.state + B.off_Q);
  uint16_t* __restrict__ Th = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qt_hi);
  uint16_t* __restrict__ Tl = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qt_lo);
  uint16_t* __restrict__ Nh = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qn_hi);
  uint16_t* __restrict__ Nl = reinterpret_cast<uint16_t*>(bs.ws + B.off_Qn_lo);
  const int a0 = it.a0, j0 = it.j0, tid = threadIdx.x;
  // read 32 rows (a) x 64 columns (j), j fastest
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = tid + 256 * i, a = id >> 6, j = id & 63;
    const bool in = a0 + a < R && j0 + j < n;
    const float x = in ? Q[(int64_t)(a0 + a) * n + j0 + j] : 0.f;
    tile[a][j] = x;
    if (in) {
      uint32_t h, l;
      split_pair(x, 0.f, h, l);
      Nh[(int64_t)(a0 + a) * n + j0 + j] = (uint16_t)h;
      Nl[(int64_t)(a0 + a) * n + j0 + j] = (uint16_t)l;
    }
  }
  __syncthreads();
  // write 64 rows (j) x 32 columns (a), a fastest
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = tid + 256 * i, j = id >> 5, a = id & 31;
    if (a0 + a < R && j0 + j < n) {
      uint32_t h, l;
      split_pair(tile[a][j], 0.f, h, l);
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
