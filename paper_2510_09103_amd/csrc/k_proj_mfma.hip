// Fused low-rank step with R held (refresh period T > 1, steps between two runs of Alg. 2).
//
// With orthonormal rows Q = R the arg-min of Alg. 1 over L alone is a projection:
//   P   = G Q^T                                  (m x r)
//   L_t = beta1 L_{t-1} + (1-beta1) P            (least-squares fit of m_t = (1-beta1) G + beta1 L_{t-1} Q)
//   m^c = G + beta1 (L_{t-1} - P) Q              (eq. 3-4 with r_t = L_t Q - m_t)
//   W  <- W - lr (clip(m^c / (sqrt(v) + eps)) + lambda W)     (Alg. 1 last line)
// One workgroup owns a stripe of 64 rows of one block and makes two passes over it:
//   pass 1 streams G (HBM, through LDS) and accumulates P on the matrix cores; the Q operand arrives
//          already laid out as MFMA fragments and goes straight from L2 into registers; row sums of
//          G^2 for the blockwise second moment ride along;
//   pass 2 re-reads G, reconstructs D Q tile by tile (D = beta1 (L_{t-1} - P), held in registers as
//          A fragments) and applies the update to W; Q^T arrives as a ready-made padded LDS image,
//          copied by direct global->LDS loads that overlap the element-wise tail of the previous tile.
// Matrix work uses v_mfma_f32_32x32x16_bf16.  G is bf16 (exact); every fp32 operand (Q, D) is
// carried as a (hi, lo) pair of bf16 values, products hi*hi + lo*hi + hi*lo accumulated in fp32
// (relative operand error 2^-17).  The two images of Q are written by qimage_kernel after each run
// of Alg. 2.  Three workgroups fit on a CU (LDS 53.8 KB, <= 168 VGPRs), so the phases of different
// stripes overlap.
#include "adapm_plan.h"
#include "ew_math.h"

namespace adapm {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 64;     // rows per stripe
constexpr int BK = 64;     // columns per chunk (both passes)
constexpr int GS = BK + 8; // LDS row stride of the G tile (elements): 16-byte fragment reads hit all banks
constexpr int CS = BK + 8; // LDS row stride of the fp32 C tile

union Frag {
  bf16x8 v;
  uint4 q;
};
__device__ __forceinline__ bf16x8 as_frag(const uint4& q) {
  Frag f;
  f.q = q;
  return f.v;
}
__device__ __forceinline__ bf16x8 lds_frag(const uint16_t* p) { return as_frag(*reinterpret_cast<const uint4*>(p)); }

// geometry of the two images of Q
__host__ __device__ constexpr int timg_row_stride(int R) { return R + 8; }                             // elements
__host__ __device__ constexpr int timg_chunk_bytes(int R) { return 2 * BK * timg_row_stride(R) * 2; }  // hi + lo
__host__ __device__ constexpr int qf_chunk_bytes(int R) { return (BK / 16) * (R / 32) * 2 * 64 * 16; }

template <int RT, bool W16>
__global__ __launch_bounds__(256, 3) void proj_kernel(const ProjItem* __restrict__ items,
                                                      const LrBlockDev* __restrict__ lrb, Bases bs, StepScalars sc) {
  constexpr int R = 32 * RT;
  constexpr int DS = timg_row_stride(R);
  constexpr int TPW = (2 * RT >= 4) ? (2 * RT / 4) : 1;   // pass-1 output tiles per wave
  constexpr int PS = R + 4;
  constexpr int G_BYTES = BM * GS * 2;
  constexpr int P_BYTES = BM * PS * 4;
  constexpr int D_BYTES = 2 * BM * DS * 2;
  constexpr int T_BYTES = timg_chunk_bytes(R);
  constexpr int P2_BYTES = T_BYTES + BM * CS * 4;
  constexpr int m1 = G_BYTES > P_BYTES ? G_BYTES : P_BYTES;
  constexpr int m2 = D_BYTES > P2_BYTES ? D_BYTES : P2_BYTES;
  constexpr int SMEM = m1 > m2 ? m1 : m2;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ float vrow[BM];
  __shared__ float rsum[BM];

  const ProjItem item = items[blockIdx.x];
  if (item.lr < 0) return;
  const LrBlockDev B = lrb[item.lr];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lh = lane >> 5;
  const int m = B.m, n = B.n, row0 = item.row0;
  const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(bs.grads[B.block]);
  char* __restrict__ W = reinterpret_cast<char*>(bs.params[B.block]);
  float* __restrict__ Lst = reinterpret_cast<float*>(bs.state + B.off_L);
  float* __restrict__ vst = reinterpret_cast<float*>(bs.state + B.off_v);
  const char* __restrict__ Qf = bs.ws + B.off_Qf;       // fragment-major image of Q (pass 1)
  const char* __restrict__ Timg = bs.ws + B.off_Timg;   // LDS image of Q^T per 64-column chunk (pass 2)

  // ------------------------------------------------------------------ pass 1: P = G Q^T
  uint16_t* Gs = reinterpret_cast<uint16_t*>(smem);               // [BM][GS]
  f32x16 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
  float ss0 = 0.f, ss1 = 0.f;                                      // sums of g^2: rows tid/8 and 32 + tid/8
  const bool p1_active = wave < 2 * RT;                           // r = 32: only two output tiles
  const int my_nt = (RT >= 4) ? wave : (wave % RT);
  const int my_mt0 = (RT >= 4) ? 0 : (wave / RT);

  uint4 ga[2], gb[2];                                              // G: two chunks ahead
  uint4 qa[BK / 16][2], qb[BK / 16][2];                            // Q fragments (hi, lo): this chunk / the next
  auto fetch_g = [&](int k0, uint4 (&dst)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      dst[i] = make_uint4(0, 0, 0, 0);
      if (row0 + row < m && k0 + c8 < n)
        dst[i] = *reinterpret_cast<const uint4*>(G + (int64_t)(row0 + row) * n + k0 + c8);
    }
  };
  // fragment (chunk c, k-step kk, r-tile, hi/lo) is 1 KB: lane l holds Q[32 tile + l%32][64 c + 16 kk + 8 (l/32) .. +7]
  auto fetch_q = [&](int k0, uint4 (&dst)[BK / 16][2]) {
    if (!p1_active) return;
    const char* base = Qf + (int64_t)(k0 / BK) * qf_chunk_bytes(R);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk)
#pragma unroll
      for (int hl = 0; hl < 2; ++hl)
        dst[kk][hl] = *reinterpret_cast<const uint4*>(base + ((((kk * RT + my_nt) * 2 + hl) * 64 + lane) << 4));
  };
  auto chunk = [&](int k0, uint4 (&gcur)[2], uint4 (&qcur)[BK / 16][2], uint4 (&qnxt)[BK / 16][2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      const uint4 q = gcur[i];
      *reinterpret_cast<uint4*>(Gs + row * GS + c8) = q;
      const float s = dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
      if (i == 0) ss0 += s; else ss1 += s;
    }
    __syncthreads();
    if (k0 + 2 * BK < n) fetch_g(k0 + 2 * BK, gcur);
    if (k0 + BK < n) fetch_q(k0 + BK, qnxt);
    if (p1_active) {
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        const int ko = kk * 16 + 8 * lh;
        const bf16x8 bh = as_frag(qcur[kk][0]), bl = as_frag(qcur[kk][1]);
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
  fetch_q(0, qa);
  for (int k0 = 0; k0 < n; k0 += 2 * BK) {
    chunk(k0, ga, qa, qb);
    if (k0 + BK < n) chunk(k0 + BK, gb, qb, qa);
  }

  // ------------------------------------------------------------------ second moment of the stripe
  // a row is covered by 8 consecutive lanes
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) { ss0 += __shfl_xor(ss0, o, 64); ss1 += __shfl_xor(ss1, o, 64); }
  if ((tid & 7) == 0) { rsum[tid >> 3] = ss0; rsum[32 + (tid >> 3)] = ss1; }

  // ------------------------------------------------------------------ L_t and D = dL L' + dP P
  // P leaves the accumulators through LDS so that L is read and written as whole rows (float4).
  float* Ps = reinterpret_cast<float*>(smem);                     // [BM][PS] fp32
  if (p1_active) {
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
        const float inv = inv_denom_exact(vn, sc.inv_debias_v, sc.inv_debias_m, sc.eps);
        for (int i = 0; i < g; ++i) vrow[r0 + i] = inv;
      }
    }
  } else if (B.v_kind == 2) {      // v finished by the statistics kernel: one value per group of rows
    if (tid < BM && row0 + tid < m)
      vrow[tid] = inv_denom_exact(vst[(row0 + tid) / B.v_group_rows], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
  }
  constexpr int LV = (BM * R / 4) / 256;                          // float4 per thread
  uint2 dhv[LV], dlv[LV];
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int id = tid + 256 * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
    float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row0 + row < m) {
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
  uint16_t* Th = reinterpret_cast<uint16_t*>(smem);               // [BK][DS]  Q^T hi   (image chunk, as stored)
  uint16_t* Tl = Th + BK * DS;                                    // [BK][DS]  Q^T lo
  float* Cs = reinterpret_cast<float*>(smem + T_BYTES);           // [BM][CS]
  const UpdCoef cf = make_coef(sc.lr, B.lr_scale, B.wd, sc.clip);
  const float ob2 = 1.f - sc.beta2;
  constexpr int WV = W16 ? 1 : 2;                                  // 16-byte pieces of W per 8 elements
  uint4 gcur[2], wcur[2][WV], gnxt[2], wnxt[2][WV];
  // asynchronous copy of one image chunk into LDS: every wave moves whole kilobytes
  auto dma_t = [&](int j0) {
    const char* src = Timg + (int64_t)(j0 / BK) * T_BYTES;
    constexpr int NI = T_BYTES / 1024;
#pragma unroll
    for (int i = 0; i < (NI + 3) / 4; ++i) {
      const int k = wave + 4 * i;
      if (k < NI)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + k * 1024 + lane * 16),
                                         (__attribute__((address_space(3))) void*)(smem + k * 1024), 16, 0, 0);
    }
  };
  auto fetch_gw = [&](int j0, uint4 (&gq)[2], uint4 (&wq)[2][WV]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      gq[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int k = 0; k < WV; ++k) wq[i][k] = make_uint4(0, 0, 0, 0);
      if (row0 + row < m && j0 + c8 < n) {
        const int64_t e = (int64_t)(row0 + row) * n + j0 + c8;
        gq[i] = *reinterpret_cast<const uint4*>(G + e);
#pragma unroll
        for (int k = 0; k < WV; ++k) wq[i][k] = *reinterpret_cast<const uint4*>(W + e * (W16 ? 2 : 4) + 16 * k);
      }
    }
  };
  dma_t(0);
  fetch_gw(0, gcur, wcur);
  for (int j0 = 0; j0 < n; j0 += BK) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");              // this chunk's image (and G, W) have landed
    __syncthreads();
    if (j0 + BK < n) fetch_gw(j0 + BK, gnxt, wnxt);
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
    if (j0 + BK < n) dma_t(j0 + BK);                               // overlaps the element-wise tail below
    // element-wise tail on 8 consecutive columns per thread
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, c8 = (id & 7) * 8;
      if (row0 + row >= m || j0 + c8 >= n) continue;
      const int64_t e = (int64_t)(row0 + row) * n + j0 + c8;
      const uint32_t gw[4] = {gcur[i].x, gcur[i].y, gcur[i].z, gcur[i].w};
      float g[8], mc[8], inv[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) { g[2 * j] = bf16lo(gw[j]); g[2 * j + 1] = bf16hi(gw[j]); }
      const float4 ca = *reinterpret_cast<const float4*>(Cs + row * CS + c8);
      const float4 cb = *reinterpret_cast<const float4*>(Cs + row * CS + c8 + 4);
      const float cc[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
      if (sc.cG == 1.f) {
#pragma unroll
        for (int j = 0; j < 8; ++j) mc[j] = fmaf(sc.cC, cc[j], g[j]);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) mc[j] = fmaf(sc.cC, cc[j], sc.cG * g[j]);
      }
      if (B.v_kind == 0) {          // per-element second moment
        float4* vp = reinterpret_cast<float4*>(vst + e);
        const float4 va = vp[0], vb = vp[1];
        float vv[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          vv[j] = sc.beta2 * vv[j] + ob2 * g[j] * g[j];
          inv[j] = inv_denom_fast(vv[j], sc.inv_debias_v, sc.inv_debias_m * cf.neg_lrs, sc.eps);   // -lr folded in
        }
        vp[0] = make_float4(vv[0], vv[1], vv[2], vv[3]);
        vp[1] = make_float4(vv[4], vv[5], vv[6], vv[7]);
      } else {
        const float x = vrow[row] * cf.neg_lrs;                     // -lr folded into the inverse denominator
#pragma unroll
        for (int j = 0; j < 8; ++j) inv[j] = x;
      }
      const float bound = -cf.neg_lrs * cf.clip;
      if (W16) {
        const uint32_t ww[4] = {wcur[i][0].x, wcur[i][0].y, wcur[i][0].z, wcur[i][0].w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          o[j] = pack_bf16x2(apply_update_scaled(bf16lo(ww[j]), mc[2 * j], inv[2 * j], bound, cf.decay),
                             apply_update_scaled(bf16hi(ww[j]), mc[2 * j + 1], inv[2 * j + 1], bound, cf.decay));
        *reinterpret_cast<uint4*>(W + e * 2) = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
        const uint32_t ww[8] = {wcur[i][0].x, wcur[i][0].y, wcur[i][0].z, wcur[i][0].w,
                                wcur[i][WV - 1].x, wcur[i][WV - 1].y, wcur[i][WV - 1].z, wcur[i][WV - 1].w};
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) w[j] = apply_update_scaled(__uint_as_float(ww[j]), mc[j], inv[j], bound, cf.decay);
        float4* wp = reinterpret_cast<float4*>(W + e * 4);
        wp[0] = make_float4(w[0], w[1], w[2], w[3]);
        wp[1] = make_float4(w[4], w[5], w[6], w[7]);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      gcur[i] = gnxt[i];
#pragma unroll
      for (int k = 0; k < WV; ++k) wcur[i][k] = wnxt[i][k];
    }
  }
}

// After Alg. 2: R (r x n fp32, state) -> the two bf16 (hi, lo) images used by proj_kernel, in the workspace.
//  * fragment-major image for pass 1: [chunk][k-step][r-tile][hi|lo][lane][8]  (see fetch_q)
//  * padded LDS image of Q^T for pass 2: [chunk][hi|lo][64 columns j][R + 8], zero beyond n and in the padding
// One workgroup per (block, 64-column chunk); a thread writes 16-byte pieces.
__global__ __launch_bounds__(256) void qimage_kernel(const QsItem* __restrict__ items,
                                                     const LrBlockDev* __restrict__ lrb, Bases bs) {
  const QsItem it = items[blockIdx.x];
  const LrBlockDev B = lrb[it.lr];
  const int n = B.n, R = B.r, RT = R / 32, c = it.c;
  const float* __restrict__ Q = reinterpret_cast<const float*>(bs.state + B.off_Q);
  char* qf = bs.ws + B.off_Qf + (int64_t)c * qf_chunk_bytes(R);
  char* ti = bs.ws + B.off_Timg + (int64_t)c * timg_chunk_bytes(R);
  const int DS = timg_row_stride(R);
  // pass-1 fragments: piece p = ((kk * RT + tile) * 2 + hl) * 64 + lane
  const int np1 = (BK / 16) * RT * 2 * 64;
  for (int p = threadIdx.x; p < np1; p += 256) {
    const int lane = p & 63, hl = (p >> 6) & 1, rest = p >> 7, tile = rest % RT, kk = rest / RT;
    const int a = 32 * tile + (lane & 31), k = c * BK + kk * 16 + 8 * (lane >> 5);
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x0 = (k + 2 * e < n) ? Q[(int64_t)a * n + k + 2 * e] : 0.f;
      const float x1 = (k + 2 * e + 1 < n) ? Q[(int64_t)a * n + k + 2 * e + 1] : 0.f;
      uint32_t h, l;
      split_pair(x0, x1, h, l);
      o[e] = hl ? l : h;
    }
    *reinterpret_cast<uint4*>(qf + (int64_t)p * 16) = make_uint4(o[0], o[1], o[2], o[3]);
  }
  // pass-2 image: piece p = (hl * BK + j) * (DS / 8) + a8 / 8
  const int np2 = 2 * BK * (DS / 8);
  for (int p = threadIdx.x; p < np2; p += 256) {
    const int a8 = (p % (DS / 8)) * 8, j = (p / (DS / 8)) % BK, hl = p / (BK * (DS / 8));
    const int col = c * BK + j;
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int a0 = a8 + 2 * e;
      const float x0 = (a0 < R && col < n) ? Q[(int64_t)a0 * n + col] : 0.f;
      const float x1 = (a0 + 1 < R && col < n) ? Q[(int64_t)(a0 + 1) * n + col] : 0.f;
      uint32_t h, l;
      split_pair(x0, x1, h, l);
      o[e] = hl ? l : h;
    }
    *reinterpret_cast<uint4*>(ti + (int64_t)p * 16) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

template <int RT>
void launch_proj_rt(bool w16, dim3 grid, const ProjItem* items, const LrBlockDev* lrb, Bases b, StepScalars sc,
                    hipStream_t s) {
  if (w16) hipLaunchKernelGGL((proj_kernel<RT, true>), grid, dim3(256), 0, s, items, lrb, b, sc);
  else hipLaunchKernelGGL((proj_kernel<RT, false>), grid, dim3(256), 0, s, items, lrb, b, sc);
}

}  // namespace

size_t proj_qf_bytes(int r, int n) { return (size_t)((n + BK - 1) / BK) * qf_chunk_bytes(r); }
size_t proj_timg_bytes(int r, int n) { return (size_t)((n + BK - 1) / BK) * timg_chunk_bytes(r); }

void launch_proj(int rt, bool w16, const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b,
                 StepScalars sc, hipStream_t s) {
  if (nitems <= 0) return;
  const dim3 grid((unsigned)nitems);
  if (rt == 1) launch_proj_rt<1>(w16, grid, items, lrb, b, sc, s);
  else if (rt == 2) launch_proj_rt<2>(w16, grid, items, lrb, b, sc, s);
  else launch_proj_rt<4>(w16, grid, items, lrb, b, sc, s);
}

void launch_qimage(const QsItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(qimage_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, lrb, b);
}

}  // namespace adapm
