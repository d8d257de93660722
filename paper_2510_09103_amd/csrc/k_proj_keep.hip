// Step with R held (refresh period T > 1, between two runs of Alg. 2) for blocks whose rows are short enough that a
// stripe of G can stay on chip between the two passes: the gradient is read from memory ONCE.
//
//   P   = G Q^T                              (m x r; Q = R with orthonormal rows)
//   L_t = beta1 L_{t-1} + (1-beta1) P        (least-squares fit of m_t with R held: the arg-min of Alg. 1 over L)
//   m^c = G + beta1 (L_{t-1} - P) Q          (eq. 3-4 with r_t = L_t Q - m_t)
//   W  <- W - lr (clip(m^c / (sqrt(v) + eps)) + lambda W)      (Alg. 1 last line)
//
// The update of a row needs the whole row of P, so G is needed twice.  The general kernel (proj_kernel, 128-row
// stripes) reads it twice; a second pass over a stripe never hits a cache while 256 workgroups stream.  Here a
// workgroup takes 64 rows of at most 1600 columns (200 KB of bf16) and its eight streaming waves keep every 16-byte
// vector of G they load in registers (25 vectors = 100 registers per lane) from pass 1 to pass 2; the kernel runs
// three waves per SIMD (one matrix-core wave, two streaming waves), which gives every wave 168 registers.  The price
// is that a copied chunk of an image of Q serves 64 rows instead of 128 (twice the image traffic from L2 per element).
//
// Roles (12 waves): waves 0-3 feed the matrix cores, waves 4-11 stream G and W and do the element-wise work; the two
// groups meet at one barrier per 64-column chunk.  Pass 1: streaming lane (row t/8, columns 8 (t%8)..) requests all of
// its vectors of G at once, stages them chunk by chunk into a three-deep LDS tile and sums their squares; matrix-core
// wave w accumulates rank tile w of P for both 32-row tiles from the fragment image of Q (direct global -> LDS copy,
// three buffers).  Then v, L_t and D = beta1 (L_{t-1} - P) (split into (hi, lo) bf16, held as A-fragments by the
// matrix-core waves, whose threads also prefetched L_{t-1} during pass 1).  Pass 2: matrix-core wave (wr, wc) builds the
// 32 x 32 tile of D Q from the swizzled image of Q^T and leaves it in LDS; the streaming waves read it as row vectors,
// take G from their registers, apply the update to W (requested four tiles ahead) and store it.
//
// Blocks served: rank class 128 (r <= 128), bf16 parameters, blockwise second moment (finished inside the stripe for
// groups of rows that divide 64, or beforehand by the statistics kernel), columns a multiple of 8 and at most 1600.
#include "k_stripe_common.h"

namespace adapm {

namespace {

constexpr int KM = 64;               // rows per stripe
constexpr int KT = 768;              // threads: 4 matrix-core waves + 8 streaming waves
constexpr int KMW = 4;               // matrix-core waves
constexpr int KMAXC = 25;            // 64-column chunks a stripe may have: 1600 columns
constexpr int KD2 = 4;               // tiles of W in flight per streaming thread in pass 2

template <int RT>
struct Keep {
  static constexpr int R = 32 * RT;
  static constexpr int PS = R + 4;                          // LDS row stride of P (floats)
  static constexpr int DS = R + 8;                          // LDS row stride of D (elements)
  static constexpr int QF = qf_chunk_bytes(R);
  static constexpr int TB = timg_chunk_bytes(R);
  static constexpr int G_TILE = KM * GS * 2;
  static constexpr int C_TILE = KM * CS * 4;
  // Copies of the images are started several rounds before their use: a round here is short (64 rows), shorter
  // than the latency of a copy from L2.
  static constexpr int NB1 = 4;                             // pass 1: buffers of the fragment image (used NB1 - 1 rounds after the copy starts)
  static constexpr int NG = 2;                              // pass 1: tiles of G (staged one round before their use)
  static constexpr int NB2 = 3;                             // pass 2: buffers of the image of Q^T (used two rounds after the copy starts)
  static constexpr int P1_BYTES = NB1 * QF + NG * G_TILE;
  static constexpr int P_BYTES = KM * PS * 4;
  static constexpr int D_BYTES = 2 * KM * DS * 2;
  static constexpr int MID_BYTES = P_BYTES + D_BYTES;       // P and D side by side
  static constexpr int P2_BYTES = NB2 * TB + 2 * C_TILE;
  static constexpr int m1 = P1_BYTES > MID_BYTES ? P1_BYTES : MID_BYTES;
  static constexpr int SMEM = m1 > P2_BYTES ? m1 : P2_BYTES;
};

template <int RT>
__global__ __launch_bounds__(KT, 1) void proj_keep_kernel(const ProjItem* __restrict__ items,
                                                          const LrBlockDev* __restrict__ lrb, Bases bs, StepScalars sc) {
  static_assert(RT == 4, "one rank tile per matrix-core wave");
  using K = Keep<RT>;
  constexpr int R = K::R, PS = K::PS, DS = K::DS, QF = K::QF, TB = K::TB, G_TILE = K::G_TILE, C_TILE = K::C_TILE, NB1 = K::NB1,
                NG = K::NG, NB2 = K::NB2;
  constexpr int P1A = NB1 - 1;                       // rounds between the start of a copy and its use, pass 1
  constexpr int CPW = QF / 1024 / KMW;               // copy instructions per matrix-core wave and image chunk (either image)
  static_assert(QF == TB, "both images have the same chunk size");
  __shared__ __attribute__((aligned(16))) unsigned char smem[K::SMEM];
  __shared__ float vrow[KM];
  __shared__ float rsum[KM];

  const ProjItem item = items[blockIdx.x];
  if (item.lr < 0) return;
  const LrBlockDev B = lrb[item.lr];
  // global gradient clipping: the method sees gs * G.  G stays exact bf16 in the matrix products; the factor goes on
  // their results (P), on the sums of squares (gs^2) and on the G term of m^c.
  const float gs = grad_scale(bs);
  sc.cG *= gs;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Roles by SIMD, not by wave index: every SIMD must get exactly one matrix-core wave (it has one matrix pipeline)
  // and two streaming waves.  At 168 registers a SIMD holds three waves, so the workgroup's twelve waves sit three
  // to a SIMD whatever order the dispatcher places them in; each wave reads which SIMD it runs on (HW_ID, bits 5:4)
  // and ranks itself among the workgroup's waves on the same SIMD.
  __shared__ int simd_of[KT / 64];
  const int simd = (int)__builtin_amdgcn_s_getreg((1 << 11) | (4 << 6) | 4) & 3;
  if (lane == 0) simd_of[wave] = simd;
  __syncthreads();
  int rank = 0, cnt[4] = {0, 0, 0, 0};
  for (int w = 0; w < KT / 64; ++w) {
    const int sw = simd_of[w];
    cnt[sw & 3] += 1;
    rank += (w < wave && sw == simd) ? 1 : 0;
  }
  int mw = simd;                                     // index within the matrix-core role
  if (cnt[0] != 3 || cnt[1] != 3 || cnt[2] != 3 || cnt[3] != 3) {   // not expected; roles by wave index then (same result, slower)
    mw = wave & 3;
    rank = wave >> 2;
  }
  rank = __builtin_amdgcn_readfirstlane(rank);
  mw = __builtin_amdgcn_readfirstlane(mw);
  const bool mrole = rank == 0;                      // matrix-core waves / streaming waves
  const int tm = mw * 64 + lane;                     // thread index within the matrix-core role (0 .. 255)
  const int ts = (2 * mw + (rank > 1 ? 1 : 0)) * 64 + lane;     // thread index within the streaming role (0 .. 511)
  const int l32 = lane & 31, lh = lane >> 5;
  const int m = B.m, n = B.n, r = B.r, row0 = item.row0;
  const int nc = (n + BK - 1) / BK;                  // n is a multiple of 8 and nc <= KMAXC (the planner sees to both)
  const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(bs.grads[B.block]);
  char* __restrict__ W = reinterpret_cast<char*>(bs.params[B.block]);
  float* __restrict__ Lst = reinterpret_cast<float*>(bs.state + B.off_L);
  float* __restrict__ vst = reinterpret_cast<float*>(bs.state + B.off_v);
  const char* __restrict__ Qf = bs.ws + B.off_Qf;
  const char* __restrict__ Timg = bs.ws + B.off_Timg;
  const unsigned rows_valid = (unsigned)(m - row0 < KM ? m - row0 : KM);
  const __amdgpu_buffer_rsrc_t rG = make_rsrc(G + (int64_t)row0 * n, rows_valid * (unsigned)n * 2u);
  const __amdgpu_buffer_rsrc_t rW = make_rsrc(W + (int64_t)row0 * n * 2, rows_valid * (unsigned)n * 2u);
  lds_u8* const lds = (lds_u8*)smem;
  const int NR1 = nc + P1A, NR2 = nc + 3;            // rounds of the two passes

  constexpr int LV = (KM * R / 4) / (KMW * 64);
  const bool vec4 = (r & 3) == 0;
  const UpdCoef cf = make_coef(sc.lr, B.lr_scale, B.wd, sc.clip);
  const float bound = -cf.neg_lrs * cf.clip;
  float* const Ps = reinterpret_cast<float*>(smem);                    // [KM][PS] fp32, between the passes
  uint16_t* const Dh = reinterpret_cast<uint16_t*>(smem + K::P_BYTES); // [KM][DS], then the lo halves
  uint16_t* const Dl = Dh + KM * DS;
  lds_u8* const Ts = lds;                             // pass 2: [NB2][TB]
  unsigned char* const Cs = smem + NB2 * TB;          // pass 2: [2][KM][CS] fp32

  // Each role runs its whole body in one branch (so that the registers of one role are not live in the other) and
  // the two meet at the same sequence of barriers: NR1 in pass 1, four around the middle part (S1 .. S4), NR2 in pass 2.
  // Everything the roles hand to each other goes through LDS, so every barrier waits for the wave's LDS traffic only
  // and leaves its global requests (the prefetched W) in flight.
  if (mrole) {
    // L_{t-1} of the stripe, requested now, used after pass 1 (8 float4 per thread, on clamped addresses);
    // row = id / (R / 4), columns 4 (id % (R / 4)) .. + 3
    float4 lraw[LV];
    if (vec4) {
#pragma unroll
      for (int i = 0; i < LV; ++i) {
        const int id = tm + KMW * 64 * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
        const bool ok = row0 + row < m && c4 < r;
        lraw[i] = *reinterpret_cast<const float4*>(Lst + (ok ? (int64_t)(row0 + row) * r + c4 : 0));
      }
    }
    // ---------------------------------------------------------------- pass 1: P = G Q^T, rank tile mw, both row tiles
    f32x16 acc[2], acl[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[t][i] = acl[t][i] = 0.f;
    {
      lds_u8* const Qs = lds;                                           // [NB1][QF]
      const unsigned gs0 = lds_addr(lds) + NB1 * QF;                    // [NG][KM][GS] bf16
      // round cc: start the copy of fragments cc, multiply chunk cc - P1A (its fragments landed a round ago, its tile
      // of G was staged in the last round)
      for (int cc = 0; cc < NR1; ++cc) {
        // always CPW copy instructions per wave, so that the wait below leaves exactly the newest NB1 - 2 copies in
        // flight; past the end the last chunk is copied again into a buffer nobody reads any more
        dma_copy<KMW>(Qf + (int64_t)(cc < nc ? cc : nc - 1) * QF, Qs + (cc % NB1) * QF, QF, mw, lane);
        if (cc >= P1A) {
          const int ch = cc - P1A;
          const unsigned qa = lds_addr(Qs) + (ch % NB1) * QF + (unsigned)((mw * 2 * 64 + lane) * 16);
          const unsigned ga = gs0 + (ch % NG) * G_TILE + (unsigned)((l32 * GS + 8 * lh) * 2);
          constexpr int NK = BK / 16;
          bf16x8 bh[2], bl[2], a0[2], a1[2];
          bh[0] = lds_frag_raw(qa);
          bl[0] = lds_frag_raw(qa + 1024);
          a0[0] = lds_frag_raw(ga);
          a1[0] = lds_frag_raw(ga + 32 * GS * 2);
#pragma unroll
          for (int kk = 0; kk < NK; ++kk) {
            const int c = kk & 1, nx = c ^ 1;
            if (kk + 1 < NK) {
              bh[nx] = lds_frag_raw(qa + (kk + 1) * RT * 2048);
              bl[nx] = lds_frag_raw(qa + (kk + 1) * RT * 2048 + 1024);
              a0[nx] = lds_frag_raw(ga + (kk + 1) * 32);
              a1[nx] = lds_frag_raw(ga + (kk + 1) * 32 + 32 * GS * 2);
              lds_wait_keep<4>(bh[c], bl[c], a0[c], a1[c]);
            } else {
              lds_wait(bh[c], bl[c], a0[c], a1[c]);
            }
            // four independent accumulation chains (row tile x hi / lo half of Q): this wave is the only one that
            // feeds its SIMD's matrix pipeline, so nothing else would cover the latency of a dependent product
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[c], bh[c], acc[1], 0, 0, 0);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bh[c], acc[0], 0, 0, 0);
            acl[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[c], bl[c], acl[1], 0, 0, 0);
            acl[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bl[c], acl[0], 0, 0, 0);
          }
        }
        if (cc + 1 < NR1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CPW * (NB1 - 2)) : "memory");   // fragments cc - (NB1 - 2) have landed
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                     // last round: nothing may still be landing
        wg_barrier();
      }
    }
    wg_barrier();                                                   // S1: the pass-1 buffers are free
    {
      const int col = 32 * mw + l32;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int p = 0; p < 4; ++p) Ps[(32 * t + 8 * q + 4 * lh + p) * PS + col] = acc[t][4 * q + p] + acl[t][4 * q + p];
    }
    wg_barrier();                                                   // S2: P is in LDS
    // ---------------------------------------------------------------- L_t and D = dL L' + dP P (whole rows, float4)
    // The kernel is compiled for the rank class R; the block's own rank r <= R sets the row stride of L.  Columns
    // r .. R-1 of P are zero (the images of Q are zero-padded), and so are those of D.
#pragma unroll
    for (int i = 0; i < LV; ++i) {
      const int id = tm + KMW * 64 * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
      float lprev[4] = {0.f, 0.f, 0.f, 0.f}, d[4] = {0.f, 0.f, 0.f, 0.f};
      if (row0 + row < m && c4 < r) {
        float* lp = Lst + (int64_t)(row0 + row) * r + c4;
        const float4 pv4 = *reinterpret_cast<const float4*>(Ps + row * PS + c4);
        const float pv[4] = {gs * pv4.x, gs * pv4.y, gs * pv4.z, gs * pv4.w};
        const float b1 = sc.beta1, ob1 = 1.f - sc.beta1;
        if (vec4) {
          const float4 t = lraw[i];
          lprev[0] = t.x; lprev[1] = t.y; lprev[2] = t.z; lprev[3] = t.w;
          *reinterpret_cast<float4*>(lp) = make_float4(b1 * lprev[0] + ob1 * pv[0], b1 * lprev[1] + ob1 * pv[1],
                                                       b1 * lprev[2] + ob1 * pv[2], b1 * lprev[3] + ob1 * pv[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c4 + e < r) { lprev[e] = lp[e]; lp[e] = b1 * lprev[e] + ob1 * pv[e]; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) d[e] = (c4 + e < r) ? sc.dL * lprev[e] + sc.dP * pv[e] : 0.f;
      }
      uint32_t h0, l0, h1, l1;
      split_pair(d[0], d[1], h0, l0);
      split_pair(d[2], d[3], h1, l1);
      *reinterpret_cast<uint2*>(Dh + row * DS + c4) = make_uint2(h0, h1);
      *reinterpret_cast<uint2*>(Dl + row * DS + c4) = make_uint2(l0, l1);
    }
    wg_barrier();                                                   // S3: D is in LDS
    // ---------------------------------------------------------------- pass 2: C = D Q
    // A fragments of D: wave (wr, wc) owns rows 32 wr .. and columns 32 wc .. of every 64 x 64 tile
    const int wr = mw & 1, wc = mw >> 1;
    bf16x8 dh[2 * RT], dl[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) {
      dh[ks] = lds_frag(lds + K::P_BYTES + ((32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
      dl[ks] = lds_frag(lds + K::P_BYTES + ((KM + 32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
    }
    wg_barrier();                                                   // S4: D is in registers, its LDS is free
    const int jl = 32 * wc + l32;                                      // column of this lane inside the tile
    unsigned toff[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) toff[ks] = (unsigned)(jl * R * 2 + timg_piece(R, jl, 2 * ks + lh) * 16);
    const int coff = (32 * wr + 4 * lh) * CS + 32 * wc + l32;          // this lane's first result inside a C tile
    // round j: start the copy of image j, build tile j-2 from the image that landed a round ago
    for (int j = 0; j < NR2; ++j) {
      dma_copy<KMW>(Timg + (int64_t)(j < nc ? j : nc - 1) * TB, Ts + (j % NB2) * TB, TB, mw, lane);
      if (j >= 2 && j < nc + 2) {
        const int tj = j - 2;
        const unsigned th = lds_addr(Ts) + (tj % NB2) * TB, tl = th + BK * R * 2;
        f32x16 c, c2;
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = c2[i] = 0.f;
        // the fragments of the next pair of k-steps are requested before the products of this pair are issued: with one
        // matrix-core wave per SIMD nothing else hides the wave's LDS latency
        bf16x8 bh0[2], bl0[2], bh1[2], bl1[2];
        bh0[0] = lds_frag_raw(th + toff[0]);
        bl0[0] = lds_frag_raw(tl + toff[0]);
        bh1[0] = lds_frag_raw(th + toff[1]);
        bl1[0] = lds_frag_raw(tl + toff[1]);
#pragma unroll
        for (int ks = 0; ks < 2 * RT; ks += 2) {
          const int cu = (ks >> 1) & 1, nx = cu ^ 1;
          if (ks + 2 < 2 * RT) {
            bh0[nx] = lds_frag_raw(th + toff[ks + 2]);
            bl0[nx] = lds_frag_raw(tl + toff[ks + 2]);
            bh1[nx] = lds_frag_raw(th + toff[ks + 3]);
            bl1[nx] = lds_frag_raw(tl + toff[ks + 3]);
            lds_wait_keep<4>(bh0[cu], bl0[cu], bh1[cu], bl1[cu]);
          } else {
            lds_wait(bh0[cu], bl0[cu], bh1[cu], bl1[cu]);
          }
          // two independent accumulation chains, added at the end (see pass 1)
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bh0[cu], c, 0, 0, 0);
          c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks], bh0[cu], c2, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bl0[cu], c, 0, 0, 0);
          c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bh1[cu], c2, 0, 0, 0);
          c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks + 1], bh1[cu], c, 0, 0, 0);
          c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bl1[cu], c2, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] += c2[i];
        lds_f32* cs = (lds_f32*)(lds + NB2 * TB + (tj & 1) * C_TILE);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int p = 0; p < 4; ++p) cs[coff + (8 * q + p) * CS] = c[4 * q + p];
      }
      if (j + 1 < NR2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CPW) : "memory");   // image j-1 has landed
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      wg_barrier();
    }
  } else {
    // ---------------------------------------------------------------- streaming role
    // this lane's vector of every chunk, kept from pass 1 to pass 2: row ts / 8, columns 8 (ts % 8) .. + 7 of the chunk
    const int srow = ts >> 3, c8 = (ts & 7) * 8;
    const unsigned eoff = (unsigned)(srow * n + c8);
    uint4 gk[KMAXC];
    // all vectors are requested at once (their registers are reserved anyway), in the order of their use
#pragma unroll
    for (int c = 0; c < KMAXC; ++c) gk[c] = buf_load16(rG, (c * BK + c8 < n) ? (eoff + (unsigned)(c * BK)) * 2u : OOB);
    float ss = 0.f;                                    // sum of squares of this lane's elements of its row
    unsigned char* const Gs = smem + NB1 * QF;
    // round cc: chunk cc - (P1A - 1) goes into the tile the matrix-core waves multiply in the next round
#pragma unroll
    for (int cc = 0; cc < KMAXC + P1A; ++cc) {
      if (cc < NR1) {
        if (cc >= P1A - 1 && cc - (P1A - 1) < KMAXC) {
          const int ch = cc - (P1A - 1);
          const uint4 q = gk[ch];
          *reinterpret_cast<uint4*>(Gs + (ch % NG) * G_TILE + (srow * GS + c8) * 2) = q;
          ss += dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
        }
        wg_barrier();
      }
    }
    // W of the first tiles of pass 2: requested before the element-wise middle part, which they overlap
    uint4 wq[KD2];
#pragma unroll
    for (int u = 0; u < KD2; ++u) wq[u] = buf_load16(rW, (u < nc && u * BK + c8 < n) ? (eoff + (unsigned)(u * BK)) * 2u : OOB);
    wg_barrier();                                                   // S1
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) ss += __shfl_xor(ss, o, 64);       // a row is covered by 8 consecutive lanes
    if ((ts & 7) == 0) rsum[srow] = ss * (gs * gs);
    wg_barrier();                                                   // S2: the rows' sums of squares are in LDS
    if (B.v_kind == 1) {             // groups of v_group_rows rows inside the stripe: finish v here
      const int g = B.v_group_rows;
      if (ts < KM / g) {
        const int r0 = ts * g;
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
    } else {                         // v finished by the statistics kernel: one value per group of rows
      if (ts < KM && row0 + ts < m)
        vrow[ts] = inv_denom_exact(vst[(row0 + ts) / B.v_group_rows], sc.inv_debias_v, sc.inv_debias_m, sc.eps);
    }
    wg_barrier();                                                   // S3: vrow is ready
    wg_barrier();                                                   // S4
    const float ninv = vrow[srow] * cf.neg_lrs;                        // -lr folded into the inverse denominator
    // round jj: tail of tile jj-3 (built in the last round): C from LDS, G from this lane's registers, W from the set
    // requested KD2 tiles ago; then W of tile jj-3+KD2 into the set just freed
#pragma unroll
    for (int jj = 0; jj < KMAXC + 3; ++jj) {
      if (jj < NR2) {
        if (jj >= 3) {
          const int j = jj - 3;
          const bool ok = j * BK + c8 < n;                             // j < nc here
          const unsigned e = eoff + (unsigned)(j * BK);
          const float* cs = reinterpret_cast<const float*>(Cs + (j & 1) * C_TILE) + srow * CS + c8;
          const float4 ca = *reinterpret_cast<const float4*>(cs);
          const float4 cb = *reinterpret_cast<const float4*>(cs + 4);
          const float cc[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
          const uint4 gq = gk[j];
          const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
          const uint4 wv = wq[j % KD2];
          const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w};
          uint32_t o[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float g0 = bf16lo(gw[k]), g1 = bf16hi(gw[k]);
            const float m0 = fmaf(sc.cC, cc[2 * k], sc.cG == 1.f ? g0 : sc.cG * g0);
            const float m1 = fmaf(sc.cC, cc[2 * k + 1], sc.cG == 1.f ? g1 : sc.cG * g1);
            o[k] = pack_bf16x2(apply_update_scaled(bf16lo(ww[k]), m0, ninv, bound, cf.decay),
                               apply_update_scaled(bf16hi(ww[k]), m1, ninv, bound, cf.decay));
          }
          buf_store16(rW, ok ? e * 2u : OOB, make_uint4(o[0], o[1], o[2], o[3]));
          const int jn = j + KD2;
          wq[j % KD2] = buf_load16(rW, (jn < nc && jn * BK + c8 < n) ? (eoff + (unsigned)(jn * BK)) * 2u : OOB);
        }
        wg_barrier();
      }
    }
  }
}

}  // namespace

// rows of a stripe and the widest block the kernel takes
int proj_keep_rows() { return KM; }
int proj_keep_max_cols() { return KMAXC * BK; }

void launch_proj_keep(const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, StepScalars sc, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL((proj_keep_kernel<4>), dim3((unsigned)nitems), dim3(KT), 0, s, items, lrb, b, sc);
}

}  // namespace adapm
