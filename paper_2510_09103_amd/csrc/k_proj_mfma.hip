// Stripe kernels of the low-rank blocks on the MFMA path.  All of them give one workgroup (16 waves) a
// stripe of 128 rows of one block: waves 0-7 feed the matrix cores, waves 8-15 stream G and W and do the
// element-wise work; the two groups hand tiles to each other through multi-buffered LDS with one
// barrier per tile, and the bf16 (hi, lo) images of the factors arrive by direct global -> LDS copies.
//
//  proj_kernel            step with R held (refresh period T > 1, between two runs of Alg. 2).  With
//                         orthonormal rows Q = R the arg-min of Alg. 1 over L alone is a projection:
//                           P   = G Q^T                              (m x r)
//                           L_t = beta1 L_{t-1} + (1-beta1) P        (least-squares fit of m_t)
//                           m^c = G + beta1 (L_{t-1} - P) Q          (eq. 3-4 with r_t = L_t Q - m_t)
//                           W  <- W - lr (clip(m^c / (sqrt(v) + eps)) + lambda W)    (Alg. 1 last line)
//                         pass 1: the streaming waves put chunk c of G into LDS (row sums of G^2 for the
//                         blockwise second moment ride along) while the matrix-core waves accumulate P on
//                         chunk c-2 from the fragment image of Q; pass 2: the matrix-core waves build
//                         tile j of D Q (D = beta1 (L_{t-1} - P) held in registers as A-fragments, Q^T
//                         from a bank-swizzled LDS image) while the streaming waves apply the update of
//                         tile j-2 to W and prefetch G, W (and a per-element v) of the next tiles.  Rows
//                         may start at any 2-byte alignment: vectors cover the columns up to the last
//                         multiple of 8, the remaining columns are done element by element.
//  stripe_kernel          pass 1 alone on two stripes (256 rows) that share every copied chunk of the
//                         image: the products G R^T and (G^T L)^T of Alg. 2 (the stripes of G^T are 256
//                         columns of G, staged as they lie in memory and read with the transposing LDS
//                         reads of gfx950), each continued by the thin
//                         products of the GD step on the factor rows behind the stripe (L (R R^T),
//                         L' (R' R^T) for L; the same with L^T L, L^T L' for R^T), so that the new factor
//                         is stored and the m x r / r x n products never leave the accumulators.
//  refresh_update_kernel  pass 2 alone with two (factor, image) pairs: the update of a step that ran Alg. 2,
//                         m^c = G + beta1/(1-beta1) (L_{t-1} R_{t-1} - L_t R_t), never storing the m x n term.
//  gram_kernel, qimage_kernel, qf_image_kernel, qt_image_kernel: the r x r products of Alg. 2 from the
//                         images (chunks shared through LDS, results also as images), the images themselves.
//
// Matrix work uses v_mfma_f32_32x32x16_bf16.  G is bf16 (exact); every fp32 operand (factors, D) is
// carried as a (hi, lo) pair of bf16 values, products hi*hi + lo*hi + hi*lo accumulated in fp32
// (relative operand error 2^-17).
#include "k_stripe_common.h"

namespace adapm {

namespace {

// pass-1 round of a matrix-core wave: start the copy of the next Q fragments, multiply one chunk
// (qs, gs: LDS byte addresses of the fragment buffer and the G tile to read)
template <int RT, int TPW>
__device__ __forceinline__ void p1_round(unsigned qs, unsigned gs, lds_u8* dst, const char* src, bool mma,
                                         f32x16 (&acc)[TPW], int my_rt, int my_mt0, int mw, int lane) {
  static_assert(TPW == 1 || TPW == 2, "tiles per wave");
  constexpr int QF = qf_chunk_bytes(32 * RT);
  dma_copy(src, dst, QF, mw, lane);
  if (mma) {
    const int l32 = lane & 31, lh = lane >> 5;
    const unsigned qa = qs + (unsigned)((my_rt * 2 * 64 + lane) * 16);
    const unsigned ga = gs + (unsigned)(((32 * my_mt0 + l32) * GS + 8 * lh) * 2);
    // the fragments of k-step kk+1 are requested before the products of k-step kk are issued, so the wave's
    // LDS latency hides behind its own matrix work (LDS results return in order: the wait leaves the newer
    // requests in flight)
    constexpr int NK = BK / 16, NF = 2 + TPW;
    bf16x8 bh[2], bl[2], a0[2], a1[2];
    bh[0] = lds_frag_raw(qa);
    bl[0] = lds_frag_raw(qa + 1024);
    a0[0] = lds_frag_raw(ga);
    if (TPW == 2) a1[0] = lds_frag_raw(ga + 32 * GS * 2);
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      const int c = kk & 1, nx = c ^ 1;
      if (kk + 1 < NK) {
        bh[nx] = lds_frag_raw(qa + (kk + 1) * RT * 2048);
        bl[nx] = lds_frag_raw(qa + (kk + 1) * RT * 2048 + 1024);
        a0[nx] = lds_frag_raw(ga + (kk + 1) * 32);
        if (TPW == 2) a1[nx] = lds_frag_raw(ga + (kk + 1) * 32 + 32 * GS * 2);
      }
      if (TPW == 2) {
        if (kk + 1 < NK) lds_wait_keep<NF>(bh[c], bl[c], a0[c], a1[c]); else lds_wait(bh[c], bl[c], a0[c], a1[c]);
        acc[TPW - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[c], bh[c], acc[TPW - 1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bh[c], acc[0], 0, 0, 0);
        acc[TPW - 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[c], bl[c], acc[TPW - 1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bl[c], acc[0], 0, 0, 0);
      } else {
        if (kk + 1 < NK) lds_wait_keep<NF>(bh[c], bl[c], a0[c]); else lds_wait(bh[c], bl[c], a0[c]);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bh[c], acc[0], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[c], bl[c], acc[0], 0, 0, 0);
      }
    }
  }
}

// pass-2 round of a matrix-core wave: start the copy of the next Q^T image, build one 32 x 32 tile of D Q
// (th: LDS byte address of the image to read; the C tile is written with ordinary stores at the end of
// the round, where the copy has to have landed anyway)
template <int RT>
__device__ __forceinline__ void p2_round(unsigned th, lds_u8* dst, lds_f32* cs, const char* src, bool copy, bool mma,
                                         const bf16x8 (&dh)[2 * RT], const bf16x8 (&dl)[2 * RT],
                                         const int (&toff)[2 * RT], int coff, int mw, int lane) {
  constexpr int R = 32 * RT;
  if (copy) dma_copy(src, dst, timg_chunk_bytes(R), mw, lane);
  if (mma) {
    const unsigned tl = th + BK * R * 2;
    f32x16 c;
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ks += 2) {
      bf16x8 bh0 = lds_frag_raw(th + toff[ks]);
      bf16x8 bl0 = lds_frag_raw(tl + toff[ks]);
      bf16x8 bh1 = lds_frag_raw(th + toff[ks + 1]);
      bf16x8 bl1 = lds_frag_raw(tl + toff[ks + 1]);
      lds_wait(bh0, bl0, bh1, bl1);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bh0, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks], bh0, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bl0, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bh1, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks + 1], bh1, c, 0, 0, 0);
      c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bl1, c, 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int p = 0; p < 4; ++p) cs[coff + (8 * q + p) * CS] = c[4 * q + p];
  }
}

// Geometry of pass 1 (shared by the held-R kernel and the stripe product of Alg. 2)
template <int RT>
struct Pass1 {
  static constexpr int R = 32 * RT;
  static constexpr int PS = R + 4;                        // LDS row stride of P (floats)
  static constexpr int QF = qf_chunk_bytes(R);
  static constexpr int G_TILE = BM * GS * 2;
  static constexpr int NB1 = 3;                           // buffers: a chunk is consumed two rounds after its copy starts
  static constexpr int BYTES = NB1 * QF + NB1 * G_TILE;   // LDS during the pass
  static constexpr int P_BYTES = BM * PS * 4;             // LDS holding P afterwards
  static constexpr int D1 = 3;                            // chunks of A in flight per streaming thread
};

// P = A Q^T for the 128 rows of A behind the range-checked buffer rG (bf16, row stride n; columns 0 .. nv-1,
// nv a multiple of 8, are covered: rows need not start on 16-byte boundaries, a row's last n mod 8 columns
// are the caller's business), Q given as its fragment image Qf.  Leaves P in LDS at smem as [BM][R + 4] fp32 (the caller has to
// __syncthreads() before reading it) and returns, in the streaming waves, this thread's sums of
// squares of its two rows of A (rows t512/8 and 64 + t512/8, columns 8 (t512 % 8) .. of every chunk).
template <int RT>
__device__ __forceinline__ void stripe_pass1(unsigned char* smem, __amdgpu_buffer_rsrc_t rG, int n, int nv,
                                             const char* __restrict__ Qf, float& ss0, float& ss1) {
  constexpr int QF = Pass1<RT>::QF, G_TILE = Pass1<RT>::G_TILE, NB1 = Pass1<RT>::NB1, PS = Pass1<RT>::PS, D1 = Pass1<RT>::D1;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool mrole = wave < 8;
  const int mw = wave & 7, t512 = tid & 511, l32 = lane & 31, lh = lane >> 5;
  const int nc = (nv + BK - 1) / BK;
  const int c8 = (t512 & 7) * 8;
  const unsigned eoff[2] = {(unsigned)((t512 >> 3) * n + c8), (unsigned)((64 + (t512 >> 3)) * n + c8)};
  const int NR1 = (nc + 1 + D1) / D1 * D1;             // rounds: nc + 2, rounded up to the prefetch depth
  // Streaming waves put chunk c of G into LDS (and sum g^2 per row) while the matrix-core waves
  // multiply chunk c-1; the Q fragments of chunk c arrive by direct-to-LDS copy.  One barrier per chunk.
  lds_u8* const lds = (lds_u8*)smem;
  lds_u8* const Qs = lds;                             // [NB1][QF]
  unsigned char* Gs = smem + NB1 * QF;                // [NB1][BM][GS] bf16
  constexpr int TPW = (4 * RT >= 8) ? (4 * RT / 8) : 1;          // output tiles per matrix-core wave
  const bool p1_active = mrole && (mw < 4 * RT);
  const int my_rt = mw % RT;                                      // r-tile
  const int my_mt0 = (mw / RT) * TPW;                             // first row tile
  f32x16 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
  ss0 = 0.f; ss1 = 0.f;
  auto fetch_g = [&](int c, uint4 (&dst)[2]) {
    const bool ok = c * BK + c8 < nv;
#pragma unroll
    for (int i = 0; i < 2; ++i) dst[i] = buf_load16(rG, ok ? (eoff[i] + (unsigned)(c * BK)) * 2u : OOB);
  };
  auto stage_g = [&](int buf, uint4 (&src)[2]) {
    uint16_t* gs = reinterpret_cast<uint16_t*>(Gs + buf * G_TILE);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = (t512 >> 3) + 64 * i;
      const uint4 q = src[i];
      *reinterpret_cast<uint4*>(gs + row * GS + c8) = q;
      const float s = dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
      if (i == 0) ss0 += s; else ss1 += s;
    }
  };
  // Both roles run NR1 rounds and meet at one barrier per round (the branch is wave-uniform).  Round cc:
  // the streaming waves stage chunk cc of G and fetch chunk cc+2; the matrix-core waves start the copy of
  // fragments cc and multiply chunk cc-2, whose G tile and fragments were completed one round ago.  Three
  // buffers of each, so nothing is waited for in the round it was started in.  The streaming loop has no
  // conditions, so the compiler can count its outstanding loads and keeps them in flight across barriers.
  if (mrole) {
    int b_cur = 0, b_mma = 1;                         // cc % NB1, (cc - 2) % NB1
    for (int cc = 0; cc < NR1; ++cc) {
      // always RT copy instructions per wave, so the wait below leaves exactly the newest copy in flight;
      // past the end the last chunk is copied again into a buffer nobody reads
      p1_round<RT, TPW>(lds_addr(Qs) + b_mma * QF, lds_addr(Qs) + NB1 * QF + b_mma * G_TILE, Qs + b_cur * QF,
                        Qf + (int64_t)(cc < nc ? cc : nc - 1) * QF, cc >= 2 && cc < nc + 2 && p1_active, acc, my_rt, my_mt0,
                        mw, lane);
      b_cur = b_cur + 1 == NB1 ? 0 : b_cur + 1;
      b_mma = b_mma + 1 == NB1 ? 0 : b_mma + 1;
      if (cc + 1 < NR1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(RT) : "memory");  // this wave's share of fragments cc-1
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                        // last round: nothing may still be landing
      wg_barrier();
    }
  } else {
    uint4 gq[D1][2];
#pragma unroll
    for (int u = 0; u < D1; ++u) {
      fetch_g(u, gq[u]);
      __builtin_amdgcn_sched_barrier(0);   // keep issue order = use order, or the loop's first wait drains everything
    }
    int buf = 0;                               // cc % NB1
    for (int cb = 0; cb < NR1; cb += D1) {     // chunks at or beyond nc read zeros into a tile nobody multiplies
#pragma unroll
      for (int u = 0; u < D1; ++u) {
        stage_g(buf, gq[u]);
        fetch_g(cb + u + D1, gq[u]);
        wg_barrier();
        buf = buf + 1 == NB1 ? 0 : buf + 1;
      }
    }
  }
  __syncthreads();
  if (p1_active) {
    float* Ps = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const int col = 32 * my_rt + l32;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = 0; p < 4; ++p) Ps[(32 * (my_mt0 + t) + 8 * q + 4 * lh + p) * PS + col] = acc[t][4 * q + p];
    }
  }
}

// Pass 1 over TWO stripes (256 rows) at once: every chunk of the fragment image of Q that is copied into LDS
// serves both, which halves the image traffic per row of A (the copies, 32 KB per 64 columns, cost more than a
// quarter of the pass at 128 rows).  Two buffers of the image and of the A tile: round cc copies fragments cc
// and stages chunk cc of A while chunk cc-1 is multiplied; the copy has to land within its round.
template <int RT>
struct Pass1x2 {
  static constexpr int R = 32 * RT;
  static constexpr int ROWS = 2 * BM;
  static constexpr int PS = R + 4;                        // LDS row stride of P (floats)
  static constexpr int QF = qf_chunk_bytes(R);
  static constexpr int G_TILE = ROWS * GS * 2;
  static constexpr int BYTES = 2 * QF + 2 * G_TILE;       // LDS during the pass
  static constexpr int P_BYTES = ROWS * PS * 4;           // LDS holding P afterwards
  static constexpr int D1 = 2;                            // chunks of A in flight per streaming thread
};

// Thin products appended to the stripe product (the GD step of Alg. 2 on one factor): P <- cp P + c1 X B1 + c2 X' B2
// for the 256 x r pieces X, X' of the factor and its predecessor that belong to the stripe's rows.
struct StripeTail {
  const float* xc;                   // X(j, a) = xc[j * sj + a * sa], j = row of the stripe; null: no tail
  const float* xp;                   // X' likewise
  int64_t sj, sa;
  int rows, r;                       // rows of the stripe that exist; columns of X
  const char* img1;                  // fragment images of B1^T, B2^T (r x r, rank class of the stripe product)
  const char* img2;
  float c1, c2, cp;
  int nmat;                          // 2, or 1: only the first thin product (X' = X and B2 = B1 folded into c1)
  char* timg;                        // non-null (nmat = 1, sj = 1): also write X (unscaled) as the image of a transposed factor,
                                     // [hi|lo][row of the stripe][R] per 64 rows, for the fused update; points at the stripe's first chunk
};

// As stripe_pass1, for the 256 rows behind rG: leaves P in LDS at smem as [256][R + 4] ([256][R + 1] with TRA) fp32 (the caller has to
// __syncthreads() before reading it); rsum (LDS, 256 floats, or null) receives the sums of squares of the rows.
// With a tail, the thin products run as further rounds of the same pipeline: the streaming waves scale a 64-column
// chunk of X by its coefficient and stage it as two bf16 tiles (hi, lo), the matrix-core waves copy the matching
// chunk of the coefficient image and multiply hi * (hi, lo) + lo * hi onto the accumulators that hold P.
// TRA = false: A is the 256 x K stripe behind rG (row stride n = K elements).  TRA = true: the stripe is 256 columns
// of a K x ld row-major matrix (base points at the stripe's first column): the stripe product of the transposed
// matrix without a transposed copy.  A chunk is then 64 rows of that matrix, staged as it lies in memory (512
// contiguous bytes per row), and the matrix-core waves take their fragments with transpose reads.
struct StripeSrc {
  __amdgpu_buffer_rsrc_t rG;         // TRA = false
  int n, nv;
  const uint16_t* base;              // TRA = true
  int64_t ld;
  int K, width;                      // rows of the matrix; columns of the stripe that exist
};
constexpr int TS = 4 * BK + 32;      // LDS row stride (elements) of a transposed-read tile: rows 64 bytes apart in bank space

template <int RT, bool TRA>
__device__ __forceinline__ void stripe_pass1_x2(unsigned char* smem, const StripeSrc& src, const char* __restrict__ Qf,
                                                float* rsum, const StripeTail& tl) {
  constexpr int QF = Pass1x2<RT>::QF, G_TILE = Pass1x2<RT>::G_TILE, D1 = Pass1x2<RT>::D1;
  constexpr int PS = TRA ? 32 * RT + 1 : Pass1x2<RT>::PS;   // row stride of P (see stripe_kernel)
  static_assert(BK * TS * 2 <= G_TILE, "a transposed-read tile fits the tile buffer");
  constexpr int TPW = RT;                                 // 8 row tiles x RT rank tiles over 8 waves
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool mrole = wave < 8;
  const int mw = wave & 7, t512 = tid & 511, l32 = lane & 31, lh = lane >> 5;
  const __amdgpu_buffer_rsrc_t rG = src.rG;
  const int n = src.n, nv = src.nv;
  const int nc = ((TRA ? src.K : nv) + BK - 1) / BK;
  const int c8 = (t512 & 7) * 8;
  unsigned eoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) eoff[i] = (unsigned)(((t512 >> 3) + 64 * i) * n + c8);
  // TRA: this thread's vectors of a chunk: rows t512 / 32 + 16 i, columns 8 (t512 % 32) .. + 7 of the stripe
  const int tj = (t512 & 31) * 8, tr = t512 >> 5;
  const int NR1 = (nc + D1) / D1 * D1;                    // rounds: nc + 1, rounded up to the prefetch depth
  lds_u8* const lds = (lds_u8*)smem;
  lds_u8* const Qs = lds;                                 // [2][QF]
  unsigned char* Gs = smem + 2 * QF;                      // [2][256][GS] bf16
  const int my_rt = mw % RT;                              // rank tile
  const int my_mt0 = (mw / RT) * TPW;                     // first of this wave's TPW row tiles
  float ss[4] = {0.f, 0.f, 0.f, 0.f};   // this streaming thread's sums of squares of rows t512 / 8 + 64 i
  auto fetch_g = [&](int c, uint4 (&dst)[4]) {
    if (TRA) {
      // the chunk's own range: rows at or beyond K read zeros; 32-bit offsets stay below 64 rows of the matrix
      const int rows = src.K - c * BK < BK ? src.K - c * BK : BK;
      const __amdgpu_buffer_rsrc_t rc = make_rsrc(src.base + (int64_t)c * BK * src.ld,
                                                  rows > 0 ? (unsigned)(((int64_t)(rows - 1) * src.ld + src.width) * 2) : 0u);
      const bool ok = tj < src.width;
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[i] = buf_load16(rc, ok ? (unsigned)((tr + 16 * i) * (int)src.ld + tj) * 2u : OOB);
    } else {
      const bool ok = c * BK + c8 < nv;
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[i] = buf_load16(rG, ok ? (eoff[i] + (unsigned)(c * BK)) * 2u : OOB);
    }
  };
  auto stage_g = [&](int buf, uint4 (&q4)[4]) {
    uint16_t* gs = reinterpret_cast<uint16_t*>(Gs + buf * G_TILE);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 q = q4[i];
      if (TRA) {
        *reinterpret_cast<uint4*>(gs + (tr + 16 * i) * TS + tj) = q;
      } else {
        const int row = (t512 >> 3) + 64 * i;
        *reinterpret_cast<uint4*>(gs + row * GS + c8) = q;
        ss[i] += dot2_sq(q.w, dot2_sq(q.z, dot2_sq(q.y, dot2_sq(q.x, 0.f))));
      }
    }
  };
  f32x16 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
  if (mrole) {
    for (int cc = 0; cc < NR1; ++cc) {
      if (cc < nc) dma_copy(Qf + (int64_t)cc * QF, Qs + (cc & 1) * QF, QF, mw, lane);
      if (cc >= 1 && cc <= nc) {
        const int b = (cc - 1) & 1;
        const unsigned qa = lds_addr(Qs) + b * QF + (unsigned)((my_rt * 2 * 64 + lane) * 16);
        const unsigned ga = lds_addr(Qs) + 2 * QF + b * G_TILE + (unsigned)(((32 * my_mt0 + l32) * GS + 8 * lh) * 2);
        // TRA: lane s of a 16-lane block addresses row 8 (lane / 32) + s / 4 (+ 4 for the second read) of the k-step,
        // columns 32 tile + 16 (lane / 16 % 2) + 4 (s % 4) .. + 3; it receives column 32 tile + lane % 32
        const unsigned gt = lds_addr(Qs) + 2 * QF + b * G_TILE +
                            (unsigned)(((8 * lh + ((lane & 15) >> 2)) * TS + 32 * my_mt0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
          bf16x8 bh = lds_frag_raw(qa + kk * RT * 2048);
          bf16x8 bl = lds_frag_raw(qa + kk * RT * 2048 + 1024);
          bf16x8 a[TPW];
          if (TRA) {
            // the halves of a fragment are put together only behind the wait that names them
            u32x2 lo[TPW], hi[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
              lo[t] = lds_tr16_raw(gt + (unsigned)((16 * kk * TS + 32 * t) * 2));
              hi[t] = lds_tr16_raw(gt + (unsigned)(((16 * kk + 4) * TS + 32 * t) * 2));
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) lds_wait(lo[t], hi[t]);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
              const u32x4 both = {lo[t].x, lo[t].y, hi[t].x, hi[t].y};
              a[t] = __builtin_bit_cast(bf16x8, both);
            }
          } else {
#pragma unroll
            for (int t = 0; t < TPW; ++t) a[t] = lds_frag_raw(ga + kk * 32 + t * 32 * GS * 2);
          }
          if (TPW == 1) lds_wait(bh, bl, a[0]);
          else {
            lds_wait(bh, bl, a[0], a[1]);
            if (TPW == 4) lds_wait(a[TPW - 2], a[TPW - 1]);
          }
#pragma unroll
          for (int t = 0; t < TPW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], bh, acc[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < TPW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], bl, acc[t], 0, 0, 0);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // fragments cc have landed
      wg_barrier();
    }
  } else {
    uint4 gq[D1][4];
#pragma unroll
    for (int u = 0; u < D1; ++u) {
      fetch_g(u, gq[u]);
      __builtin_amdgcn_sched_barrier(0);   // keep issue order = use order, or the loop's first wait drains everything
    }
    static_assert(D1 % 2 == 0, "the A tile buffer of round cb + u is u % 2");
    for (int cb = 0; cb < NR1; cb += D1) {   // chunks at or beyond nc read zeros into a tile nobody multiplies
#pragma unroll
      for (int u = 0; u < D1; ++u) {
        stage_g(u & 1, gq[u]);
        fetch_g(cb + u + D1, gq[u]);
        wg_barrier();
      }
    }
    if (rsum) {                               // a row is covered by 8 consecutive lanes
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) ss[i] += __shfl_xor(ss[i], o, 64);
        if ((t512 & 7) == 0) rsum[(t512 >> 3) + 64 * i] = ss[i];
      }
    }
  }
  if (tl.xc) {
    // Every round above ended with a barrier behind its reads, so both tile buffers and both image buffers are free.
    // Chunk q = (matrix, 64 columns of X): barrier A = tiles staged and image landed, barrier B = both read.  The
    // tail moves about as many bytes per stripe as a short stripe product does and runs at that rate; deeper
    // prefetching of its operands (measured) gains nothing.
    const int nk2 = (tl.r + BK - 1) / BK, nq = tl.nmat * nk2;
    if (mrole) {
      dma_copy(tl.img1, Qs, QF, mw, lane);
#pragma unroll
      for (int t = 0; t < TPW; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] *= tl.cp;
      const unsigned g_hi = lds_addr(Qs) + 2 * QF + (unsigned)(((32 * my_mt0 + l32) * GS + 8 * lh) * 2);
      const unsigned g_lo = g_hi + G_TILE;
      for (int q = 0; q < nq; ++q) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        wg_barrier();
        if (q + 1 < nq)
          dma_copy((q + 1 < nk2 ? tl.img1 + (int64_t)(q + 1) * QF : tl.img2 + (int64_t)(q + 1 - nk2) * QF),
                   Qs + ((q + 1) & 1) * QF, QF, mw, lane);
        const unsigned qa = lds_addr(Qs) + (q & 1) * QF + (unsigned)((my_rt * 2 * 64 + lane) * 16);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
          bf16x8 bh = lds_frag_raw(qa + kk * RT * 2048);
          bf16x8 bl = lds_frag_raw(qa + kk * RT * 2048 + 1024);
          bf16x8 a[TPW];
#pragma unroll
          for (int t = 0; t < TPW; ++t) a[t] = lds_frag_raw(g_hi + kk * 32 + t * 32 * GS * 2);
          if (TPW == 1) lds_wait(bh, bl, a[0]);
          else {
            lds_wait(bh, bl, a[0], a[1]);
            if (TPW == 4) lds_wait(a[TPW - 2], a[TPW - 1]);
          }
#pragma unroll
          for (int t = 0; t < TPW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], bh, acc[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < TPW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], bl, acc[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < TPW; ++t) a[t] = lds_frag_raw(g_lo + kk * 32 + t * 32 * GS * 2);
          if (TPW == 1) lds_wait(bh, a[0]);
          else {
            lds_wait(bh, a[0], a[1]);
            if (TPW == 4) lds_wait(a[TPW - 2], a[TPW - 1]);
          }
#pragma unroll
          for (int t = 0; t < TPW; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], bh, acc[t], 0, 0, 0);
        }
        wg_barrier();
      }
    } else {
      // this thread's slots: rows t512 / 8 + 64 i, columns c8 .. c8 + 7 of the chunk.  Range-checked loads on 32-bit
      // offsets: a slot outside the piece of X reads zeros or a neighbouring element of X, and is masked when staged
      const bool vec = tl.sa == 1 && (tl.r & 3) == 0 && (tl.sj & 3) == 0;
      const unsigned xbytes = (unsigned)(((int64_t)(tl.rows - 1) * tl.sj + (int64_t)(tl.r - 1) * tl.sa + 1) * 4);
      const __amdgpu_buffer_rsrc_t rXc = make_rsrc(tl.xc, xbytes), rXp = make_rsrc(tl.xp, xbytes);
      const unsigned sj4 = (unsigned)tl.sj * 4u, sa4 = (unsigned)tl.sa * 4u;
      float raw[4][8];
      auto fetch_x = [&](int q) {
        const __amdgpu_buffer_rsrc_t rX = q < nk2 ? rXc : rXp;
        const unsigned k0 = (unsigned)((q < nk2 ? q : q - nk2) * BK + c8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned at = (unsigned)((t512 >> 3) + 64 * i) * sj4 + k0 * sa4;
          if (vec) {
            const uint4 u = buf_load16(rX, at), v = buf_load16(rX, at + 16u);
            raw[i][0] = __uint_as_float(u.x); raw[i][1] = __uint_as_float(u.y);
            raw[i][2] = __uint_as_float(u.z); raw[i][3] = __uint_as_float(u.w);
            raw[i][4] = __uint_as_float(v.x); raw[i][5] = __uint_as_float(v.y);
            raw[i][6] = __uint_as_float(v.z); raw[i][7] = __uint_as_float(v.w);
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              raw[i][e] = __uint_as_float((unsigned)__builtin_amdgcn_raw_buffer_load_b32(rX, (int)(at + (unsigned)e * sa4), 0, 0));
          }
        }
      };
      fetch_x(0);
      uint16_t* const t_hi = reinterpret_cast<uint16_t*>(Gs);
      uint16_t* const t_lo = reinterpret_cast<uint16_t*>(Gs + G_TILE);
      for (int q = 0; q < nq; ++q) {
        const float cf = q < nk2 ? tl.c1 : tl.c2;
        const int k0 = (q < nk2 ? q : q - nk2) * BK + c8;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = (t512 >> 3) + 64 * i;
          uint32_t h[4], l[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float x0 = (row < tl.rows && k0 + 2 * e < tl.r) ? cf * raw[i][2 * e] : 0.f;
            const float x1 = (row < tl.rows && k0 + 2 * e + 1 < tl.r) ? cf * raw[i][2 * e + 1] : 0.f;
            split_pair(x0, x1, h[e], l[e]);
          }
          *reinterpret_cast<uint4*>(t_hi + row * GS + c8) = make_uint4(h[0], h[1], h[2], h[3]);
          *reinterpret_cast<uint4*>(t_lo + row * GS + c8) = make_uint4(l[0], l[1], l[2], l[3]);
        }
        if (TRA && tl.timg) {
          // the thread holds 8 consecutive columns of X for one row of the stripe: one 16-byte piece of that row of
          // the transposed image (rows beyond the stripe's end inside its last 64-row chunk are written as zeros)
          constexpr int pr = 32 * RT / 8;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int row = (t512 >> 3) + 64 * i;
            if (k0 / 8 < pr && (row & ~(BK - 1)) < tl.rows) {
              uint32_t uh[4], ul[4];
#pragma unroll
              for (int e = 0; e < 4; ++e)
                split_pair((row < tl.rows && k0 + 2 * e < tl.r) ? raw[i][2 * e] : 0.f,
                           (row < tl.rows && k0 + 2 * e + 1 < tl.r) ? raw[i][2 * e + 1] : 0.f, uh[e], ul[e]);
              const int jc = row & (BK - 1);
              char* dst = tl.timg + (int64_t)(row / BK) * timg_chunk_bytes(32 * RT) +
                          ((int64_t)jc * pr + timg_piece(32 * RT, jc, k0 / 8)) * 16;
              *reinterpret_cast<uint4*>(dst) = make_uint4(uh[0], uh[1], uh[2], uh[3]);
              *reinterpret_cast<uint4*>(dst + (int64_t)BK * pr * 16) = make_uint4(ul[0], ul[1], ul[2], ul[3]);
            }
          }
        }
        wg_barrier();
        if (q + 1 < nq) fetch_x(q + 1);
        wg_barrier();
      }
    }
  }
  __syncthreads();
  if (mrole) {
    float* Ps = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
      const int col = 32 * my_rt + l32;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = 0; p < 4; ++p) Ps[(32 * (my_mt0 + t) + 8 * q + 4 * lh + p) * PS + col] = acc[t][4 * q + p];
    }
  }
}

template <int RT, bool W16, bool VEL>
__global__ __launch_bounds__(NT, 1) void proj_kernel(const ProjItem* __restrict__ items,
                                                     const LrBlockDev* __restrict__ lrb, Bases bs, StepScalars sc) {
  constexpr int R = 32 * RT;
  constexpr int DS = R + 8;                               // LDS row stride of D (elements)
  constexpr int PS = R + 4;                               // LDS row stride of P (floats)
  constexpr int TB = timg_chunk_bytes(R);
  constexpr int C_TILE = BM * CS * 4;
  constexpr int P1_BYTES = Pass1<RT>::BYTES;
  constexpr int P_BYTES = Pass1<RT>::P_BYTES;
  constexpr int D_BYTES = 2 * BM * DS * 2;
  constexpr int P2_BYTES = 2 * TB + 2 * C_TILE;
  constexpr int m1 = P1_BYTES > P_BYTES ? P1_BYTES : P_BYTES;
  constexpr int m2 = D_BYTES > P2_BYTES ? D_BYTES : P2_BYTES;
  constexpr int SMEM = m1 > m2 ? m1 : m2;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ float vrow[BM];
  __shared__ float rsum[BM];
  __shared__ float ctail[BM * 8];                         // (D Q) of a row's last n mod 8 columns

  const ProjItem item = items[blockIdx.x];
  if (item.lr < 0) return;
  const LrBlockDev B = lrb[item.lr];
  // global gradient clipping: the method sees gs * G.  G stays exact bf16 in the matrix products; the factor
  // goes on their results (P), on the sums of squares (gs^2) and on the G term of m^c.
  const float gs = grad_scale(bs);
  sc.cG *= gs;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool mrole = wave < 8;                       // matrix-core waves / streaming waves
  const int mw = wave & 7;                           // index within the role
  const int t512 = tid & 511;                        // thread index within the role
  const int l32 = lane & 31, lh = lane >> 5;
  const int m = B.m, n = B.n, row0 = item.row0;
  // Rows of G and W need not start on 16-byte boundaries (n need not be a multiple of 8): the 8-element vectors
  // of the two passes cover columns 0 .. n8-1 of every row at whatever alignment they have; the last
  // n mod 8 columns of the rows are done element by element beside the passes (rank-(n mod 8) correction of P,
  // their share of D Q, their update).
  const int n8 = n & ~7, nt = n - n8;
  const int nc = (n8 + BK - 1) / BK;
  const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(bs.grads[B.block]);
  char* __restrict__ W = reinterpret_cast<char*>(bs.params[B.block]);
  float* __restrict__ Lst = reinterpret_cast<float*>(bs.state + B.off_L);
  float* __restrict__ vst = reinterpret_cast<float*>(bs.state + B.off_v);
  const char* __restrict__ Qf = bs.ws + B.off_Qf;
  const char* __restrict__ Timg = bs.ws + B.off_Timg;
  // the stripe's rows of G and W as range-checked buffers; this thread's two 8-element vectors per
  // 64-column chunk sit in rows t512/8 and 64 + t512/8 at columns 8 (t512 % 8) ..
  constexpr unsigned WE = W16 ? 2 : 4;
  const unsigned rows_valid = (unsigned)(m - row0 < BM ? m - row0 : BM);
  const __amdgpu_buffer_rsrc_t rG = make_rsrc(G + (int64_t)row0 * n, rows_valid * (unsigned)n * 2u);
  const __amdgpu_buffer_rsrc_t rW = make_rsrc(W + (int64_t)row0 * n * WE, rows_valid * (unsigned)n * WE);
  // VEL (every block of the launch has a per-element second moment): the stripe's rows of v as a third
  // range-checked buffer, prefetched with G and W
  const __amdgpu_buffer_rsrc_t rV = make_rsrc(vst + (VEL ? (int64_t)row0 * n : 0), VEL ? rows_valid * (unsigned)n * 4u : 0u);
  const int c8 = (t512 & 7) * 8;
  const unsigned eoff[2] = {(unsigned)((t512 >> 3) * n + c8), (unsigned)((64 + (t512 >> 3)) * n + c8)};
  // rounds of pass 2: nc + 2, rounded up to the prefetch depth of the streaming waves (their loop is
  // unrolled by the depth so that every register set has a fixed name)
  constexpr int D2 = (W16 && !VEL) ? 3 : 2;          // tiles of G and W (and v) in flight per thread
  const int NR2 = (nc + 1 + D2) / D2 * D2;

  // ------------------------------------------------------------------ pass 1: P = G Q^T, left in LDS
  float ss0, ss1;                                    // streaming thread: sums of g^2 of rows t512/8 and 64 + t512/8
  stripe_pass1<RT>(smem, rG, n, n8, Qf, ss0, ss1);
  lds_u8* const lds = (lds_u8*)smem;

  // ------------------------------------------------------------------ second moment of the stripe, P to LDS
  const float* Ps = reinterpret_cast<const float*>(smem);         // [BM][PS] fp32
  if (!mrole) {                     // a row is covered by 8 consecutive lanes
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) { ss0 += __shfl_xor(ss0, o, 64); ss1 += __shfl_xor(ss1, o, 64); }
    if ((t512 & 7) == 0) { rsum[t512 >> 3] = ss0 * (gs * gs); rsum[64 + (t512 >> 3)] = ss1 * (gs * gs); }
  }
  __syncthreads();
  // the last n mod 8 columns: their G and Q (fp32, exact) staged beside P, then P += G_tail Q_tail^T and the
  // rows' sums of squares
  constexpr int TAIL_OFF = (P_BYTES > D_BYTES ? P_BYTES : D_BYTES);
  static_assert(TAIL_OFF % 16 == 0 && TAIL_OFF + (BM + R) * 8 * 4 <= SMEM, "tail staging fits beside P and D");
  float* const gtail = reinterpret_cast<float*>(smem + TAIL_OFF);   // [BM][8]
  float* const qtail = gtail + BM * 8;                              // [R][8]
  if (nt > 0) {
    const float* __restrict__ Qst = reinterpret_cast<const float*>(bs.state + B.off_Q);   // r x n
    for (int id = tid; id < (BM + R) * 8; id += NT) {
      const int c = id & 7;
      float x = 0.f;
      if (id < BM * 8) {
        const int row = id >> 3;
        if (c < nt && row0 + row < m) x = bf16lo((uint32_t)G[(int64_t)(row0 + row) * n + n8 + c]);
      } else {
        const int k = (id >> 3) - BM;
        if (c < nt && k < B.r) x = Qst[(int64_t)k * n + n8 + c];
      }
      gtail[id] = x;
    }
    __syncthreads();
    float* Pw = reinterpret_cast<float*>(smem);
    for (int id = tid; id < BM * R; id += NT) {
      const int row = id / R, k = id % R;
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) acc = fmaf(gtail[row * 8 + c], qtail[k * 8 + c], acc);
      Pw[row * PS + k] += acc;
    }
    if (tid < BM) {
      float q = 0.f;
#pragma unroll
      for (int c = 0; c < 8; ++c) q = fmaf(gtail[tid * 8 + c], gtail[tid * 8 + c], q);
      rsum[tid] += q * (gs * gs);
    }
    __syncthreads();
  }
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
  // ------------------------------------------------------------------ L_t and D = dL L' + dP P (whole rows, float4)
  // The kernel is compiled for the rank class R; the block's own rank r <= R sets the row stride of L.
  // Columns r .. R-1 of P are zero (the images of Q are zero-padded), and so are those of D.
  constexpr int LV = (BM * R / 4) / NT;
  const int r = B.r;
  const bool vec4 = (r & 3) == 0;
  uint2 dhv[LV], dlv[LV];
  // the thread's vectors of L_{t-1} are requested together, on clamped (valid) addresses, before any of them is
  // replaced: a load behind the previous vector's store would wait for it (four latencies per stripe)
  float4 lraw[LV];
  if (vec4) {
#pragma unroll
    for (int i = 0; i < LV; ++i) {
      const int id = tid + NT * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
      const bool ok = row0 + row < m && c4 < r;
      lraw[i] = *reinterpret_cast<const float4*>(Lst + (ok ? (int64_t)(row0 + row) * r + c4 : 0));
    }
  }
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int id = tid + NT * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
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
    dhv[i] = make_uint2(h0, h1);
    dlv[i] = make_uint2(l0, l1);
  }
  __syncthreads();                                                 // Ps is dead, D takes its place
  uint16_t* Dh = reinterpret_cast<uint16_t*>(smem);               // [BM][DS]
  uint16_t* Dl = Dh + BM * DS;
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    const int id = tid + NT * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
    *reinterpret_cast<uint2*>(Dh + row * DS + c4) = dhv[i];
    *reinterpret_cast<uint2*>(Dl + row * DS + c4) = dlv[i];
  }
  __syncthreads();
  if (nt > 0) {                    // (D Q) of the last n mod 8 columns, kept until the end of pass 2
    static_assert(BM * 8 == NT, "one tail element per thread");
    const int row = tid >> 3, c = tid & 7;
    float acc = 0.f;
    for (int k = 0; k < R; ++k)
      acc = fmaf(bf16lo((uint32_t)Dh[row * DS + k]) + bf16lo((uint32_t)Dl[row * DS + k]), qtail[k * 8 + c], acc);
    ctail[tid] = acc;
  }
  // ------------------------------------------------------------------ pass 2: C = D Q, update W
  // Matrix-core waves build tile j of D Q (Q^T image j came by direct-to-LDS copy during tile j-1) while
  // the streaming waves run the element-wise tail of tile j-1 and prefetch G, W.  One barrier per tile.
  lds_u8* const Ts = lds;                             // [2][TB]
  unsigned char* Cs = smem + 2 * TB;                  // [2][BM][CS] fp32
  const UpdCoef cf = make_coef(sc.lr, B.lr_scale, B.wd, sc.clip);
  const float ob2 = (1.f - sc.beta2) * (gs * gs);                  // per-element v sees (gs g)^2
  const float bound = -cf.neg_lrs * cf.clip;
  constexpr int WV = W16 ? 1 : 2;                                  // 16-byte pieces of W per 8 elements
  // Pass 2 walks the stripe from its last 64-column chunk to its first: tile j of the loops is chunk nc-1-j,
  // so what pass 1 read last is asked for again first and part of the second read of G is served by the caches.
  constexpr int VV = VEL ? 2 : 1;                                  // 16-byte pieces of v per 8 elements (VEL only)
  auto fetch_gw = [&](int j, uint4 (&gq)[2], uint4 (&wq)[2][WV], uint4 (&vq)[2][VV]) {
    const int pj = nc - 1 - j;
    const bool ok = (unsigned)pj < (unsigned)nc && pj * BK + c8 < n8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const unsigned e = eoff[i] + (unsigned)(pj * BK);
      gq[i] = buf_load16(rG, ok ? e * 2u : OOB);
#pragma unroll
      for (int k = 0; k < WV; ++k) wq[i][k] = buf_load16(rW, ok ? e * WE + 16u * k : OOB);
      if (VEL) {
#pragma unroll
        for (int k = 0; k < VV; ++k) vq[i][k] = buf_load16(rV, ok ? e * 4u + 16u * k : OOB);
      }
    }
  };
  // tile j < 0 or at / beyond nc: every store falls outside the buffer and is dropped
  auto tail = [&](int j, uint4 (&gq)[2], uint4 (&wq)[2][WV], uint4 (&vq)[2][VV]) {
    const float* cs = reinterpret_cast<const float*>(Cs + (j & 1) * C_TILE);
    const int pj = nc - 1 - j;
    const bool ok = (unsigned)pj < (unsigned)nc && pj * BK + c8 < n8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = (t512 >> 3) + 64 * i;
      const unsigned e = eoff[i] + (unsigned)(pj * BK);
      const uint32_t gw[4] = {gq[i].x, gq[i].y, gq[i].z, gq[i].w};
      float g[8], mc[8], inv[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) { g[2 * k] = bf16lo(gw[k]); g[2 * k + 1] = bf16hi(gw[k]); }
      const float4 ca = *reinterpret_cast<const float4*>(cs + row * CS + c8);
      const float4 cb = *reinterpret_cast<const float4*>(cs + row * CS + c8 + 4);
      const float cc[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
      if (sc.cG == 1.f) {
#pragma unroll
        for (int k = 0; k < 8; ++k) mc[k] = fmaf(sc.cC, cc[k], g[k]);
      } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) mc[k] = fmaf(sc.cC, cc[k], sc.cG * g[k]);
      }
      if (VEL) {                    // per-element second moment, its old values prefetched with G and W
        const uint32_t vw[8] = {vq[i][0].x, vq[i][0].y, vq[i][0].z, vq[i][0].w,
                                vq[i][VV - 1].x, vq[i][VV - 1].y, vq[i][VV - 1].z, vq[i][VV - 1].w};
        float vv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          vv[k] = sc.beta2 * __uint_as_float(vw[k]) + ob2 * g[k] * g[k];
          inv[k] = inv_denom_fast(vv[k], sc.inv_debias_v, sc.inv_debias_m * cf.neg_lrs, sc.eps);   // -lr folded in
        }
        buf_store16(rV, ok ? e * 4u : OOB, make_uint4(__float_as_uint(vv[0]), __float_as_uint(vv[1]), __float_as_uint(vv[2]), __float_as_uint(vv[3])));
        buf_store16(rV, ok ? e * 4u + 16u : OOB, make_uint4(__float_as_uint(vv[4]), __float_as_uint(vv[5]), __float_as_uint(vv[6]), __float_as_uint(vv[7])));
      } else {
        const float x = vrow[row] * cf.neg_lrs;                     // -lr folded into the inverse denominator
#pragma unroll
        for (int k = 0; k < 8; ++k) inv[k] = x;
      }
      if (W16) {
        const uint32_t ww[4] = {wq[i][0].x, wq[i][0].y, wq[i][0].z, wq[i][0].w};
        uint32_t o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
          o[k] = pack_bf16x2(apply_update_scaled(bf16lo(ww[k]), mc[2 * k], inv[2 * k], bound, cf.decay),
                             apply_update_scaled(bf16hi(ww[k]), mc[2 * k + 1], inv[2 * k + 1], bound, cf.decay));
        buf_store16(rW, ok ? e * 2u : OOB, make_uint4(o[0], o[1], o[2], o[3]));
      } else {
        const uint32_t ww[8] = {wq[i][0].x, wq[i][0].y, wq[i][0].z, wq[i][0].w,
                                wq[i][WV - 1].x, wq[i][WV - 1].y, wq[i][WV - 1].z, wq[i][WV - 1].w};
        uint32_t w[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
          w[k] = __float_as_uint(apply_update_scaled(__uint_as_float(ww[k]), mc[k], inv[k], bound, cf.decay));
        buf_store16(rW, ok ? e * 4u : OOB, make_uint4(w[0], w[1], w[2], w[3]));
        buf_store16(rW, ok ? e * 4u + 16u : OOB, make_uint4(w[4], w[5], w[6], w[7]));
      }
    }
  };
  if (mrole) {
    // A fragments of D: wave (wr, wc) owns rows 32 wr .. and columns 32 wc .. of every 128 x 64 tile
    const int wr = mw & 3, wc = mw >> 2;
    bf16x8 dh[2 * RT], dl[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) {
      dh[ks] = lds_frag(lds + ((32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
      dl[ks] = lds_frag(lds + ((BM + 32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
    }
    __syncthreads();                                               // D is in registers, its LDS is free
    const int jl = 32 * wc + l32;                                  // column of this lane inside the tile
    int toff[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) toff[ks] = jl * R * 2 + timg_piece(R, jl, 2 * ks + lh) * 16;
    const int coff = (32 * wr + 4 * lh) * CS + 32 * wc + l32;      // this lane's first result inside a C tile
    // round j: start the copy of image j, build tile j-1 from the image that landed in the last round
    for (int j = 0; j < NR2; ++j) {
      p2_round<RT>(lds_addr(Ts) + ((j - 1) & 1) * TB, Ts + (j & 1) * TB, (lds_f32*)(lds + 2 * TB + ((j - 1) & 1) * C_TILE),
                   Timg + (int64_t)(j < nc ? nc - 1 - j : 0) * TB, j < nc, j >= 1 && j <= nc, dh, dl, toff, coff, mw, lane);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // image j has landed
      wg_barrier();
    }
  } else {
    uint4 gq[D2][2], wq[D2][2][WV], vq[D2][2][VV];                 // G / W (/ v) vectors of D2 tiles in flight
#pragma unroll
    for (int u = 0; u < D2; ++u)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        gq[u][i] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int k = 0; k < WV; ++k) wq[u][i][k] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int k = 0; k < VV; ++k) vq[u][i][k] = make_uint4(0, 0, 0, 0);
      }
    __syncthreads();
#pragma unroll
    for (int u = 0; u + 2 < D2; ++u) {                             // tiles the loop does not fetch itself
      fetch_gw(u, gq[u], wq[u], vq[u]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // round j: tail of tile j-2 (built in the last round) from register set (j-2) % D2, then fetch tile
    // j-2+D2 into the set just freed.  No conditions in the loop, so the loads of the next tiles stay in
    // flight across the barriers.
    for (int jb = 0; jb < NR2; jb += D2) {
#pragma unroll
      for (int u = 0; u < D2; ++u) {
        const int su = (u + 2 * D2 - 2) % D2;
        tail(jb + u - 2, gq[su], wq[su], vq[su]);
        fetch_gw(jb + u - 2 + D2, gq[su], wq[su], vq[su]);
        wg_barrier();
      }
    }
  }
  // ------------------------------------------------------------------ the last n mod 8 columns, one element per thread
  if (nt > 0) {
    const int row = tid >> 3, c = tid & 7;
    if (c < nt && row0 + row < m) {
      const int64_t e = (int64_t)(row0 + row) * n + n8 + c;
      const float g = bf16lo((uint32_t)G[e]);
      const float mc = fmaf(sc.cC, ctail[tid], sc.cG == 1.f ? g : sc.cG * g);
      float inv;
      if (VEL) {
        const float vv = sc.beta2 * vst[e] + ob2 * g * g;
        vst[e] = vv;
        inv = inv_denom_fast(vv, sc.inv_debias_v, sc.inv_debias_m * cf.neg_lrs, sc.eps);
      } else {
        inv = vrow[row] * cf.neg_lrs;
      }
      if (W16) {
        uint16_t* wp = reinterpret_cast<uint16_t*>(W) + e;
        *wp = (uint16_t)pack_bf16x2(apply_update_scaled(bf16lo((uint32_t)*wp), mc, inv, bound, cf.decay), 0.f);
      } else {
        float* wp = reinterpret_cast<float*>(W) + e;
        *wp = apply_update_scaled(*wp, mc, inv, bound, cf.decay);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Images of a factor Q(a, k) = q[a * s0 + k * s1] (fp32, rows x K, rows <= R): one workgroup builds one
// 64-column chunk.  The chunk is read once, along whichever index is contiguous in memory, into an LDS tile
// (every load on a clamped index, masked afterwards); each 16-byte piece of an image is then cut from the tile
// and written with its (hi, lo) partner by one thread.
constexpr int QT_LD = BK + 1;                      // LDS row stride of the tile (floats)

template <int R>
__device__ __forceinline__ void q_tile_load(float* tile, const float* __restrict__ Q, int64_t s0, int64_t s1,
                                            int rows, int K, int c) {
  const int k0 = c * BK;
  if (s1 == 1) {                                   // rows of Q are contiguous: lanes run along k
    for (int id = threadIdx.x; id < R * BK; id += 256) {
      const int a = id / BK, k = id % BK;
      const bool ok = a < rows && k0 + k < K;
      const float x = Q[ok ? (int64_t)a * s0 + (k0 + k) : 0];
      tile[a * QT_LD + k] = ok ? x : 0.f;
    }
  } else {                                         // columns are contiguous (a transposed view): lanes run along a
    for (int id = threadIdx.x; id < R * BK; id += 256) {
      const int k = id / R, a = id % R;
      const bool ok = a < rows && k0 + k < K;
      const float x = Q[ok ? (int64_t)a * s0 + (int64_t)(k0 + k) * s1 : 0];
      tile[a * QT_LD + k] = ok ? x : 0.f;
    }
  }
}

// pass-1 fragment image of the chunk: [k-step][r-tile][hi|lo][lane][8]; lane l holds Q[32 tile + l%32][16 kk + 8 (l/32) .. +7]
template <int R>
__device__ __forceinline__ void q_tile_fragments(const float* tile, char* qf) {
  constexpr int RT = R / 32;
  constexpr int np = (BK / 16) * RT * 64;          // (hi, lo) pairs of pieces
  for (int p = threadIdx.x; p < np; p += 256) {
    const int lane = p & 63, rest = p >> 6, tl = rest % RT, kk = rest / RT;
    const float* src = tile + (32 * tl + (lane & 31)) * QT_LD + kk * 16 + 8 * (lane >> 5);
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_pair(src[2 * e], src[2 * e + 1], h[e], l[e]);
    char* dst = qf + ((int64_t)((kk * RT + tl) * 2) * 64 + lane) * 16;
    *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
    *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(l[0], l[1], l[2], l[3]);
  }
}

// pass-2 image of the chunk: [hi|lo][column j][R]; logical piece q (8 consecutive rows of Q) of column j sits at
// physical piece timg_piece(R, j, q)
template <int R>
__device__ __forceinline__ void q_tile_transposed(const float* tile, char* ti) {
  constexpr int pr = R / 8;
  for (int p = threadIdx.x; p < BK * pr; p += 256) {
    const int q = p % pr, j = p / pr;
    const float* src = tile + (8 * q) * QT_LD + j;
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_pair(src[(2 * e) * QT_LD], src[(2 * e + 1) * QT_LD], h[e], l[e]);
    char* dst = ti + ((int64_t)j * pr + timg_piece(R, j, q)) * 16;
    *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
    *reinterpret_cast<uint4*>(dst + (int64_t)BK * pr * 16) = make_uint4(l[0], l[1], l[2], l[3]);
  }
}

// After Alg. 2: R (r x n fp32, state) -> the two bf16 (hi, lo) images used by proj_kernel, in the workspace.
// One workgroup per (block, 64-column chunk); a thread writes 16-byte pieces.
template <int R>
__device__ __forceinline__ void q_images(float* tile, const float* __restrict__ Q, int64_t s0, int64_t s1, int rows, int K, int c,
                                         char* qf, char* ti) {
  q_tile_load<R>(tile, Q, s0, s1, rows, K, c);
  __syncthreads();
  if (qf) q_tile_fragments<R>(tile, qf + (int64_t)c * qf_chunk_bytes(R));
  if (ti) q_tile_transposed<R>(tile, ti + (int64_t)c * timg_chunk_bytes(R));
}
__device__ __forceinline__ void q_images_rc(int rc, float* tile, const float* __restrict__ Q, int64_t s0, int64_t s1, int rows,
                                            int K, int c, char* qf, char* ti) {
  if (rc == 32) q_images<32>(tile, Q, s0, s1, rows, K, c, qf, ti);
  else if (rc == 64) q_images<64>(tile, Q, s0, s1, rows, K, c, qf, ti);
  else q_images<128>(tile, Q, s0, s1, rows, K, c, qf, ti);
}

__global__ __launch_bounds__(256) void qimage_kernel(const QsItem* __restrict__ items,
                                                     const LrBlockDev* __restrict__ lrb, Bases bs) {
  __shared__ float tile[128 * QT_LD];
  const QsItem it = items[blockIdx.x];
  const LrBlockDev B = lrb[it.lr];                                      // rows r .. rc-1 of both images are zero
  q_images_rc(B.rc, tile, reinterpret_cast<const float*>(bs.state + B.off_Q), B.n, 1, B.r, B.n, it.c, bs.ws + B.off_Qf,
              bs.ws + B.off_Timg);
}

// ---------------------------------------------------------------------------------------------------
// Fused update of a step that ran Alg. 2: W <- update(m^c), m^c = cG G + cC (a1 L1 Q1 + a2 L2 Q2), one
// workgroup per 128-row stripe.  The rank-2r term is built tile by tile and never stored (eq. 3-4 fused
// into the last line of Alg. 1).  Rounds of 32 columns: matrix-core wave (wr, p) holds rows 32 wr .. of
// a_p L_p as A-fragments and builds the 32 x 32 tile of product p from the image of Q_p^T (copied
// global -> LDS without registers, two buffers); the streaming waves add the two partial tiles, apply the
// update and keep G, W of the next tiles in flight.
template <bool W16>
struct RuTail {
  // one 8-element vector of a row: columns col .. col+7 of the stripe
  static __device__ __forceinline__ void run(const float (&c)[8], const uint4& gq, const uint4 (&wq)[W16 ? 1 : 2],
                                             bool ok, unsigned e, __amdgpu_buffer_rsrc_t rW, float* vp, bool v_elem,
                                             float vinv, const StepScalars& sc, const UpdCoef& cf, float bound, float gs2) {
    const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w};
    float g[8], mc[8], inv[8];
#pragma unroll
    for (int k = 0; k < 4; ++k) { g[2 * k] = bf16lo(gw[k]); g[2 * k + 1] = bf16hi(gw[k]); }
#pragma unroll
    for (int k = 0; k < 8; ++k) mc[k] = fmaf(sc.cC, c[k], sc.cG * g[k]);
    if (v_elem) {                   // per-element second moment
      float vv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (ok) {
        const f32x4_a4 va = reinterpret_cast<const f32x4_a4*>(vp)[0], vb = reinterpret_cast<const f32x4_a4*>(vp)[1];
        vv[0] = va.x; vv[1] = va.y; vv[2] = va.z; vv[3] = va.w;
        vv[4] = vb.x; vv[5] = vb.y; vv[6] = vb.z; vv[7] = vb.w;
      }
      const float ob2 = (1.f - sc.beta2) * gs2;                    // v sees the clipped gradient
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        vv[k] = sc.beta2 * vv[k] + ob2 * g[k] * g[k];
        inv[k] = inv_denom_fast(vv[k], sc.inv_debias_v, sc.inv_debias_m * cf.neg_lrs, sc.eps);   // -lr folded in
      }
      if (ok) {
        reinterpret_cast<f32x4_a4*>(vp)[0] = f32x4_a4{vv[0], vv[1], vv[2], vv[3]};
        reinterpret_cast<f32x4_a4*>(vp)[1] = f32x4_a4{vv[4], vv[5], vv[6], vv[7]};
      }
    } else {
#pragma unroll
      for (int k = 0; k < 8; ++k) inv[k] = vinv;                    // -lr already folded in
    }
    if (W16) {
      const uint32_t ww[4] = {wq[0].x, wq[0].y, wq[0].z, wq[0].w};
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        o[k] = pack_bf16x2(apply_update_scaled(bf16lo(ww[k]), mc[2 * k], inv[2 * k], bound, cf.decay),
                           apply_update_scaled(bf16hi(ww[k]), mc[2 * k + 1], inv[2 * k + 1], bound, cf.decay));
      buf_store16(rW, ok ? e * 2u : OOB, make_uint4(o[0], o[1], o[2], o[3]));
    } else {
      const uint32_t ww[8] = {wq[0].x, wq[0].y, wq[0].z, wq[0].w, wq[W16 ? 0 : 1].x, wq[W16 ? 0 : 1].y, wq[W16 ? 0 : 1].z,
                              wq[W16 ? 0 : 1].w};
      uint32_t w[8];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        w[k] = __float_as_uint(apply_update_scaled(__uint_as_float(ww[k]), mc[k], inv[k], bound, cf.decay));
      buf_store16(rW, ok ? e * 4u : OOB, make_uint4(w[0], w[1], w[2], w[3]));
      buf_store16(rW, ok ? e * 4u + 16u : OOB, make_uint4(w[4], w[5], w[6], w[7]));
    }
  }
};

template <int RT, bool W16>
__global__ __launch_bounds__(NT, 1) void refresh_update_kernel(const ProjItem* __restrict__ items,
                                                               const RuBlockDev* __restrict__ blocks, Bases bs,
                                                               StepScalars sc) {
  constexpr int R = 32 * RT;
  constexpr int DS = R + 8;                       // LDS row stride of the staged factors (elements)
  constexpr int BR = 32;                          // columns per round
  constexpr int CR = BR + 8;                      // LDS row stride of a partial C tile (floats)
  constexpr int TH = BR * R * 2;                  // bytes of one (hi or lo) half of a round's image of one product
  constexpr int TP = 2 * TH;                      // ... of one product
  constexpr int TBUF = 2 * TP;                    // ... of one round (both products)
  constexpr int T64 = timg_chunk_bytes(R);        // the images are stored in 64-column chunks [hi|lo][64][R]
  constexpr int C_TILE = BM * CR * 4;
  constexpr int D_ONE = BM * DS * 2;              // one of (hi, lo) of one staged factor
  constexpr int D_BYTES = 4 * D_ONE;
  constexpr int P2_BYTES = 2 * TBUF + 4 * C_TILE;
  constexpr int SMEM = D_BYTES > P2_BYTES ? D_BYTES : P2_BYTES;
  constexpr int WV = W16 ? 1 : 2;
  constexpr unsigned WE = W16 ? 2 : 4;
  constexpr int D2 = 4;                           // tiles of G and W in flight per streaming thread
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  __shared__ float vrow[BM];
  __shared__ float ctail[BM * 8];                 // a1 L1 Q1 + a2 L2 Q2 of a row's last n mod 8 columns

  const ProjItem item = items[blockIdx.x];
  if (item.lr < 0) return;
  const RuBlockDev B = blocks[item.lr];
  const float gs = grad_scale(bs);                // global gradient clipping: the method sees gs * G
  sc.cG *= gs;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool mrole = wave < 8;
  const int mw = wave & 7, t512 = tid & 511, l32 = lane & 31, lh = lane >> 5;
  const int m = B.m, n = B.n, r = B.r, row0 = item.row0;
  // 8-element vectors cover columns 0 .. n8-1 of every row at whatever alignment the rows have; the last
  // n mod 8 columns are done element by element (as in the held-R kernel)
  const int n8 = n & ~7, nt = n - n8;
  const int nr = (n8 + BR - 1) / BR;              // 32-column tiles
  const int NR = (nr + 1 + D2) / D2 * D2;         // rounds: nr + 2, rounded up to the prefetch depth
  const uint16_t* __restrict__ G = reinterpret_cast<const uint16_t*>(bs.grads[B.block]);
  char* __restrict__ W = reinterpret_cast<char*>(bs.params[B.block]);
  float* __restrict__ vst = reinterpret_cast<float*>(bs.state + B.off_v);
  lds_u8* const lds = (lds_u8*)smem;

  if (B.v_kind != 0 && tid < BM && row0 + tid < m)
    vrow[tid] = inv_denom_exact(vst[(row0 + tid) / B.v_group_rows], sc.inv_debias_v, sc.inv_debias_m, sc.eps);

  // ------------------------------------------------------------------ a_p L_p -> bf16 (hi, lo) in LDS -> A-fragments
  {
    const bool vec4 = (r & 3) == 0;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const float* __restrict__ Lp = reinterpret_cast<const float*>(resolve(p == 0 ? B.l1 : B.l2, bs));
      const float a = p == 0 ? B.a1 : B.a2;
      uint16_t* Dh = reinterpret_cast<uint16_t*>(smem + (2 * p) * D_ONE);
      uint16_t* Dl = reinterpret_cast<uint16_t*>(smem + (2 * p + 1) * D_ONE);
#pragma unroll
      for (int i = 0; i < (BM * R / 4) / NT; ++i) {
        const int id = tid + NT * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
        float d[4] = {0.f, 0.f, 0.f, 0.f};
        if (row0 + row < m && c4 < r && a != 0.f) {
          const float* lp = Lp + (int64_t)(row0 + row) * r + c4;
          if (vec4) {
            const float4 t = *reinterpret_cast<const float4*>(lp);
            d[0] = a * t.x; d[1] = a * t.y; d[2] = a * t.z; d[3] = a * t.w;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (c4 + e < r) d[e] = a * lp[e];
          }
        }
        uint32_t h0, l0, h1, l1;
        split_pair(d[0], d[1], h0, l0);
        split_pair(d[2], d[3], h1, l1);
        *reinterpret_cast<uint2*>(Dh + row * DS + c4) = make_uint2(h0, h1);
        *reinterpret_cast<uint2*>(Dl + row * DS + c4) = make_uint2(l0, l1);
      }
    }
  }
  __syncthreads();
  if (nt > 0) {                    // the factors are staged: their product with the last columns of Q1, Q2
    static_assert(BM * 8 == NT, "one tail element per thread");
    const int row = tid >> 3, c = tid & 7;
    float acc = 0.f;
    if (c < nt) {
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        if ((p == 0 ? B.a1 : B.a2) == 0.f) continue;
        const float* __restrict__ Qp = reinterpret_cast<const float*>(resolve(p == 0 ? B.q1 : B.q2, bs)) + n8 + c;
        const uint16_t* Dh = reinterpret_cast<const uint16_t*>(smem + (2 * p) * D_ONE) + row * DS;
        const uint16_t* Dl = reinterpret_cast<const uint16_t*>(smem + (2 * p + 1) * D_ONE) + row * DS;
        for (int k = 0; k < r; ++k)
          acc = fmaf(bf16lo((uint32_t)Dh[k]) + bf16lo((uint32_t)Dl[k]), Qp[(int64_t)k * n], acc);
      }
    }
    ctail[tid] = acc;
  }

  unsigned char* Cs = smem + 2 * TBUF;            // [2 buffers][2 products][BM][CR] fp32
  const UpdCoef cf = make_coef(sc.lr, B.lr_scale, B.wd, sc.clip);
  const float bound = -cf.neg_lrs * cf.clip;
  if (mrole) {
    const int wr = mw & 3, prod = mw >> 2;
    bf16x8 dh[2 * RT], dl[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) {
      dh[ks] = lds_frag(lds + (2 * prod) * D_ONE + ((32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
      dl[ks] = lds_frag(lds + (2 * prod + 1) * D_ONE + ((32 * wr + l32) * DS + 16 * ks + 8 * lh) * 2);
    }
    __syncthreads();                               // the factors are in registers, their LDS is free
    // fragment offsets inside one half-image: row = column l32 of the tile; the swizzle of the stored image
    // depends on the column inside its 64-column chunk, which agrees with l32 in the bits it uses
    unsigned toff[2 * RT];
#pragma unroll
    for (int ks = 0; ks < 2 * RT; ++ks) toff[ks] = (unsigned)(l32 * R * 2 + timg_piece(R, l32, 2 * ks + lh) * 16);
    const int coff = (32 * wr + 4 * lh) * CR + l32;
    const char* img[2] = {bs.ws + B.off_img1, bs.ws + B.off_img2};
    // a product with coefficient 0 (no bias correction: a1 = 0) has no image: it is neither copied nor
    // multiplied (0 x stale bits could be NaN), its partial tile is written as zeros
    const bool live[2] = {B.a1 != 0.f, B.a2 != 0.f};
    for (int j = 0; j < NR; ++j) {
      // round j: start the copies of tile j (hi and lo halves of both products: 4 pieces of TH bytes shared
      // by the eight waves), build tile j-1 from what landed in the last round
      if (j < nr) {
        for (int k = mw; k < 4 * TH / 1024; k += 8) {
          const int q = k / (TH / 1024), piece = k % (TH / 1024);     // q = 2 * product + (lo half)
          if (!live[q >> 1]) continue;
          const char* src = img[q >> 1] + (int64_t)(j >> 1) * T64 + (q & 1) * (BK * R * 2) + (j & 1) * TH + piece * 1024;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + lane * 16),
                                           (__attribute__((address_space(3))) void*)(lds + (j & 1) * TBUF + q * TH + piece * 1024),
                                           16, 0, 0);
        }
      }
      if (j >= 1 && j <= nr) {
        const unsigned th = lds_addr(lds) + ((j - 1) & 1) * TBUF + prod * TP, tl = th + TH;
        f32x16 c;
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = 0.f;
        if (live[prod]) {
#pragma unroll
          for (int ks = 0; ks < 2 * RT; ks += 2) {
            bf16x8 bh0 = lds_frag_raw(th + toff[ks]);
            bf16x8 bl0 = lds_frag_raw(tl + toff[ks]);
            bf16x8 bh1 = lds_frag_raw(th + toff[ks + 1]);
            bf16x8 bl1 = lds_frag_raw(tl + toff[ks + 1]);
            lds_wait(bh0, bl0, bh1, bl1);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bh0, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks], bh0, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks], bl0, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bh1, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dl[ks + 1], bh1, c, 0, 0, 0);
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dh[ks + 1], bl1, c, 0, 0, 0);
          }
        }
        lds_f32* cs = (lds_f32*)(lds + 2 * TBUF + (((j - 1) & 1) * 2 + prod) * C_TILE);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int p = 0; p < 4; ++p) cs[coff + (8 * q + p) * CR] = c[4 * q + p];
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");            // the images of tile j have landed
      wg_barrier();
    }
  } else {
    // G and W are requested 64 columns (two rounds) at a time, so that a row is read and written in pieces of 128
    // bytes (64-byte pieces reach 12 - 14 % less of the memory's bandwidth): this thread owns 8-element vectors of
    // rows t512 / 8 and t512 / 8 + 64 at columns 8 (t512 % 8) .. of every 64-column pair of tiles, and finishes
    // them in the round of the pair's first or second tile, whichever holds its columns
    const unsigned rows_valid = (unsigned)(m - row0 < BM ? m - row0 : BM);
    const __amdgpu_buffer_rsrc_t rG = make_rsrc(G + (int64_t)row0 * n, rows_valid * (unsigned)n * 2u);
    const __amdgpu_buffer_rsrc_t rW = make_rsrc(W + (int64_t)row0 * n * WE, rows_valid * (unsigned)n * WE);
    const int rowa = t512 >> 3, c8 = (t512 & 7) * 8, hh = (t512 >> 2) & 1;
    const unsigned eoff[2] = {(unsigned)(rowa * n + c8), (unsigned)((rowa + 64) * n + c8)};
    const bool v_elem = B.v_kind == 0;
    static_assert(D2 == 4, "two pairs of tiles in flight");
    uint4 gq[2][2], wq[2][2][WV];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        gq[u][h] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int k = 0; k < WV; ++k) wq[u][h][k] = make_uint4(0, 0, 0, 0);
      }
    auto fetch = [&](int s, uint4 (&g)[2], uint4 (&w)[2][WV]) {     // pair s = tiles 2 s and 2 s + 1
      const bool ok = s * 64 + c8 < n8;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const unsigned e = eoff[h] + (unsigned)(s * 64);
        g[h] = buf_load16(rG, ok ? e * 2u : OOB);
#pragma unroll
        for (int k = 0; k < WV; ++k) w[h][k] = buf_load16(rW, ok ? e * WE + 16u * k : OOB);
      }
    };
    __syncthreads();
    const float vinv[2] = {v_elem ? 0.f : vrow[rowa] * cf.neg_lrs, v_elem ? 0.f : vrow[rowa + 64] * cf.neg_lrs};
    fetch(0, gq[0], wq[0]);
    __builtin_amdgcn_sched_barrier(0);
    // round jb + u: tail of tile j = jb + u - 2 (pair j / 2, register set (j / 2) % 2) by the lanes that hold its
    // columns; behind the pair's second tile, pair j / 2 + 2 is requested into the same set
    for (int jb = 0; jb < NR; jb += D2) {
#pragma unroll
      for (int u = 0; u < D2; ++u) {
        const int j = jb + u - 2, s = (jb >> 1) - 1 + (u >> 1), su = (1 + (u >> 1)) & 1;
        if (hh == (u & 1)) {
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int row = rowa + 64 * h;
            const bool ok = j >= 0 && s * 64 + c8 < n8 && row0 + row < m;
            const float* ca = reinterpret_cast<const float*>(Cs + ((j & 1) * 2) * C_TILE) + row * CR + (c8 & 31);
            const float* cb = ca + C_TILE / 4;
            const float4 a0 = *reinterpret_cast<const float4*>(ca), a1 = *reinterpret_cast<const float4*>(ca + 4);
            const float4 b0 = *reinterpret_cast<const float4*>(cb), b1 = *reinterpret_cast<const float4*>(cb + 4);
            const float c[8] = {a0.x + b0.x, a0.y + b0.y, a0.z + b0.z, a0.w + b0.w, a1.x + b1.x, a1.y + b1.y, a1.z + b1.z, a1.w + b1.w};
            const unsigned e = eoff[h] + (unsigned)(s * 64);
            RuTail<W16>::run(c, gq[su][h], wq[su][h], ok, e, rW, vst + (int64_t)row0 * n + e, v_elem, vinv[h], sc, cf, bound, gs * gs);
          }
        }
        if (u & 1) fetch(s + 2, gq[su], wq[su]);
        wg_barrier();
      }
    }
  }
  if (nt > 0) {                    // the last n mod 8 columns, one element per thread
    const int row = tid >> 3, c = tid & 7;
    if (c < nt && row0 + row < m) {
      const int64_t e = (int64_t)(row0 + row) * n + n8 + c;
      const float g = bf16lo((uint32_t)G[e]);
      const float mc = fmaf(sc.cC, ctail[tid], sc.cG * g);
      float inv;
      if (B.v_kind == 0) {
        const float vv = sc.beta2 * vst[e] + (1.f - sc.beta2) * (gs * gs) * g * g;
        vst[e] = vv;
        inv = inv_denom_fast(vv, sc.inv_debias_v, sc.inv_debias_m * cf.neg_lrs, sc.eps);
      } else {
        inv = vrow[row] * cf.neg_lrs;
      }
      if (W16) {
        uint16_t* wp = reinterpret_cast<uint16_t*>(W) + e;
        *wp = (uint16_t)pack_bf16x2(apply_update_scaled(bf16lo((uint32_t)*wp), mc, inv, bound, cf.decay), 0.f);
      } else {
        float* wp = reinterpret_cast<float*>(W) + e;
        *wp = apply_update_scaled(*wp, mc, inv, bound, cf.decay);
      }
    }
  }
}

// Image of Q^T for the fused updates: per 64-column chunk [hi|lo][column j][R], 16-byte pieces of a row
// XOR-swizzled (timg_piece); Q(a, k) = q[a * s0 + k * s1], rows r .. R-1 zero.
__global__ __launch_bounds__(256) void qt_image_kernel(const ImgItem* __restrict__ items, Bases bs) {
  __shared__ float tile[128 * QT_LD];
  const ImgItem it = items[blockIdx.x];
  q_images_rc(it.rc, tile, reinterpret_cast<const float*>(resolve(it.q.ref, bs)), it.q.s0, it.q.s1, it.r, it.K, it.c, nullptr,
              bs.ws + it.off_img);
}

// Alg. 2 stripe product: Out = A Q^T for 256 rows of A per workgroup (pass 1 of the kernel above, then a store), or
// the whole GD step on the factor behind those rows (the stripe product continued by the thin products, then a store).
// TRA: the stripes of a transposed_out problem are 256 columns of its matrix A^T (K x M, row-major: the gradient
// itself where A = G^T), read with transposing LDS reads instead of from a transposed copy.
template <int RT, bool TRA>
__global__ __launch_bounds__(NT, 1) void stripe_kernel(const StripeItem* __restrict__ items,
                                                       const StripeProb* __restrict__ probs, Bases bs) {
  // row stride of P in LDS: with the transposed store the lanes of a wave walk down a column of P, which an odd
  // stride spreads over all banks
  constexpr int R = 32 * RT, PS = TRA ? R + 1 : Pass1x2<RT>::PS, ROWS = Pass1x2<RT>::ROWS;
  constexpr int SMEM = Pass1x2<RT>::BYTES > Pass1x2<RT>::P_BYTES ? Pass1x2<RT>::BYTES : Pass1x2<RT>::P_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
  const StripeItem item = items[blockIdx.x];
  if (item.prob < 0) return;
  const StripeProb P = probs[item.prob];
  const int M = P.M, K = P.K, row0 = item.row0, tid = threadIdx.x;
  const uint16_t* __restrict__ A = reinterpret_cast<const uint16_t*>(resolve(P.a, bs));
  const unsigned rows_valid = (unsigned)(M - row0 < ROWS ? M - row0 : ROWS);
  StripeSrc src = {};
  if (TRA) {
    src.base = A + row0; src.ld = M; src.K = K; src.width = (int)rows_valid;
  } else {
    src.rG = make_rsrc(A + (int64_t)row0 * K, rows_valid * (unsigned)K * 2u);
    src.n = K; src.nv = K;
  }
  __shared__ float rsum[ROWS];        // sums of squares of the stripe's rows (second moment)
  const int r = P.r;                  // rows of Q actually present (the image is zero-padded to R)
  float gs = grad_scale(bs);          // global gradient clipping: A is the gradient (or its transpose)
  const float gs2 = gs * gs;
  // fused GD step of Alg. 2: the factor X in the layout of Out; its coefficients take the step normaliser, the one of
  // the stripe product also the gradient scale (the store below then adds X instead of scaling)
  StripeTail tl = {};
  const float* Xc = nullptr;        // may be the very buffer Out points at (iterations after the first update in place)
  if (P.upd) {
    const float s = P.off_s >= 0 ? (float)*reinterpret_cast<const double*>(bs.ws + P.off_s) : 1.f;
    Xc = reinterpret_cast<const float*>(resolve(P.x_cur, bs));
    const float* Xp = reinterpret_cast<const float*>(resolve(P.x_prev, bs));
    tl.sj = P.transpose_out ? 1 : r;
    tl.sa = P.transpose_out ? M : 1;
    tl.xc = Xc + (int64_t)row0 * tl.sj;
    tl.xp = Xp + (int64_t)row0 * tl.sj;
    tl.rows = (int)rows_valid; tl.r = r;
    tl.img1 = bs.ws + P.off_b1; tl.img2 = bs.ws + P.off_b2;
    tl.c1 = s * P.c1; tl.c2 = s * P.c2; tl.cp = s * gs * P.cp;
    tl.nmat = 2;
    // first GD iteration: the factor is still the one of the previous step and the two r x r matrices are one and the
    // same product (the Gram kernel writes it to both places), so the two thin products fold into one
    if (P.x_cur.space == P.x_prev.space && P.x_cur.off == P.x_prev.off) { tl.c1 += tl.c2; tl.nmat = 1; }
    if (TRA && tl.nmat == 1 && P.off_timg_prev >= 0)
      tl.timg = bs.ws + P.off_timg_prev + (int64_t)(row0 / BK) * timg_chunk_bytes(R);
    gs = 1.f;
  }
  stripe_pass1_x2<RT, TRA>(smem, src, bs.ws + P.off_img, (!TRA && P.v_rows > 0) ? rsum : nullptr, tl);
  __syncthreads();
  if (P.v_rows > 0) {               // groups of v_rows rows inside the stripe (v_rows divides 128)
    const int g = P.v_rows;
    if (tid < ROWS / g && row0 + tid * g < M) {
      double s = 0.0;
      for (int i = 0; i < g; ++i) s += (double)rsum[tid * g + i];
      float* vp = reinterpret_cast<float*>(bs.state + P.off_v) + (row0 + tid * g) / g;
      *vp = (float)((double)P.beta2 * (double)*vp + (1.0 - (double)P.beta2) * ((double)gs2 * s / ((double)g * (double)K)));
    }
  }
  float* Ps = reinterpret_cast<float*>(smem);
  float* Out = reinterpret_cast<float*>(bs.ws + P.off_out);
  // with the GD step, the new factor values (zeros outside the factor) go back into P for the image below
  const bool emit_f = P.upd && P.off_next >= 0, emit_t = P.upd && P.off_timg >= 0, emit = emit_f || emit_t;
  if (!P.transpose_out) {
    const bool vec4 = (r & 3) == 0;
#pragma unroll
    for (int i = 0; i < (ROWS * R / 4) / NT; ++i) {
      const int id = tid + NT * i, row = id / (R / 4), c4 = (id % (R / 4)) * 4;
      float4 v = *reinterpret_cast<const float4*>(Ps + row * PS + c4);
      float x[4] = {v.x * gs, v.y * gs, v.z * gs, v.w * gs};
      if (row0 + row < M && c4 < r) {
        const int64_t at = (int64_t)(row0 + row) * r + c4;
        float* o = Out + at;
        if (vec4) {
          if (Xc) {
            const float4 xc = *reinterpret_cast<const float4*>(Xc + at);
            x[0] += xc.x; x[1] += xc.y; x[2] += xc.z; x[3] += xc.w;
          }
          *reinterpret_cast<float4*>(o) = make_float4(x[0], x[1], x[2], x[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (c4 + e < r) {
              if (Xc) x[e] += Xc[at + e];
              o[e] = x[e];
            } else {
              x[e] = 0.f;
            }
          }
        }
      } else {
        x[0] = x[1] = x[2] = x[3] = 0.f;
      }
      if (emit) *reinterpret_cast<float4*>(Ps + row * PS + c4) = make_float4(x[0], x[1], x[2], x[3]);
    }
  } else {
    // Out[a][row0 + j] = P[j][a], four consecutive j (16 bytes) of one a per access.  A wave covers 4 values of a x 64
    // values of j: 256 contiguous bytes per a in memory, and with the odd row stride of P its 64 lanes fall on 64
    // different LDS banks.  The elements of the old factor are requested together, on clamped (valid) addresses,
    // before any of them is used.  (M is a multiple of 8 here: the stripes take only such blocks.)
    constexpr int NI = (ROWS / 4) * R / NT;
    const int j4 = 64 * ((tid >> 6) & 3) + 4 * (tid & 15), a0 = 4 * (tid >> 8) + ((tid >> 4) & 3);
    const bool jok = row0 + j4 < M;
    const int64_t col = row0 + (jok ? j4 : 0);        // columns of the factor that exist
    float4 xo[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) xo[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (Xc) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int a = a0 + 4 * (NT / 256) * i;
        xo[i] = *reinterpret_cast<const float4*>(Xc + (int64_t)(a < r ? a : 0) * M + col);
      }
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int a = a0 + 4 * (NT / 256) * i;
      float* ps = Ps + j4 * PS + a;
      float4 v = make_float4(gs * ps[0] + xo[i].x, gs * ps[PS] + xo[i].y, gs * ps[2 * PS] + xo[i].z, gs * ps[3 * PS] + xo[i].w);
      if (jok && a < r) *reinterpret_cast<float4*>(Out + (int64_t)a * M + col) = v;
      else v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (emit) { ps[0] = v.x; ps[PS] = v.y; ps[2 * PS] = v.z; ps[3 * PS] = v.w; }
    }
  }
  if (emit) __syncthreads();
  if (emit_t) {
    // image of the new factor's transpose for the fused update (the layout qt_image_kernel writes): one row of R
    // values per stripe row, its 16-byte pieces swizzled with the row's index inside the 64-row chunk
    constexpr int pr = R / 8, T64 = timg_chunk_bytes(R);
    for (int p = tid; p < ROWS * pr; p += NT) {
      const int q = p % pr, j = p / pr;
      if (row0 + (j & ~(BK - 1)) >= M) continue;   // the image ends with the chunk that holds row M - 1
      const float* src = Ps + j * PS + 8 * q;
      uint32_t h[4], l[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) split_pair(src[2 * e], src[2 * e + 1], h[e], l[e]);
      const int jc = j & (BK - 1);
      char* dst = bs.ws + P.off_timg + (int64_t)((row0 + j) / BK) * T64 + ((int64_t)jc * pr + timg_piece(R, jc, q)) * 16;
      *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
      *reinterpret_cast<uint4*>(dst + (int64_t)BK * pr * 16) = make_uint4(l[0], l[1], l[2], l[3]);
    }
  }
  if (emit_f) {
    // fragment image of the new factor for the next GD iteration (the layout qf_image_kernel writes): the stripe's
    // rows are the image's contraction index, four 64-wide chunks; lane l of a piece holds rows 16 kk + 8 (l / 32) .. + 7
    // of the chunk at factor column 32 tile + l % 32
    constexpr int QF = qf_chunk_bytes(R);
    char* const img = bs.ws + P.off_next + (int64_t)(row0 / BK) * QF;
    for (int p = tid; p < (ROWS / BK) * (BK / 16) * RT * 64; p += NT) {
      const int lane = p & 63, rest = p >> 6, tile = rest % RT, kk = (rest / RT) % (BK / 16), cq = rest / (RT * (BK / 16));
      if (row0 + BK * cq >= M) continue;          // the image ends with the chunk that holds row M - 1
      const float* src = Ps + (BK * cq + 16 * kk + 8 * (lane >> 5)) * PS + 32 * tile + (lane & 31);
      uint32_t h[4], l[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) split_pair(src[(2 * e) * PS], src[(2 * e + 1) * PS], h[e], l[e]);
      char* dst = img + (int64_t)cq * QF + ((int64_t)((kk * RT + tile) * 2) * 64 + lane) * 16;
      *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
      *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(l[0], l[1], l[2], l[3]);
    }
  }
}

// Fragment image of Q(a, k) = q[a * s0 + k * s1] (fp32, r x K): per 64-column chunk
// [k-step][r-tile][hi|lo][lane][8]; lane l holds Q[32 tile + l%32][64 c + 16 kk + 8 (l/32) .. +7].
__global__ __launch_bounds__(256) void qf_image_kernel(const ImgItem* __restrict__ items, Bases bs) {
  const ImgItem it = items[blockIdx.x];
  const int R = it.rc, RT = R / 32, K = it.K, c = it.c, rows = it.r;
  const float* __restrict__ Q = reinterpret_cast<const float*>(resolve(it.q.ref, bs));
  const int64_t s0 = it.q.s0, s1 = it.q.s1;
  char* qf = bs.ws + it.off_img + (int64_t)c * qf_chunk_bytes(R);
  const int np = (BK / 16) * RT * 64;                 // (hi, lo) pairs of pieces
  for (int p = threadIdx.x; p < np; p += 256) {
    const int lane = p & 63, rest = p >> 6, tile = rest % RT, kk = rest / RT;
    const int a = 32 * tile + (lane & 31), k = c * BK + kk * 16 + 8 * (lane >> 5);
    // the lane's 8 values: every load on a clamped (valid) index, masked afterwards; whole 16-byte vectors where
    // the rows of Q are contiguous and aligned
    float x[8];
    const bool rowok = a < rows;
    const float* qa = Q + (int64_t)(rowok ? a : 0) * s0;
    if (s1 == 1 && (s0 & 3) == 0 && (K & 3) == 0) {
      const float4 u = *reinterpret_cast<const float4*>(qa + (k < K ? k : 0));
      const float4 v = *reinterpret_cast<const float4*>(qa + (k + 4 < K ? k + 4 : 0));
      const bool ou = rowok && k < K, ov = rowok && k + 4 < K;
      x[0] = ou ? u.x : 0.f; x[1] = ou ? u.y : 0.f; x[2] = ou ? u.z : 0.f; x[3] = ou ? u.w : 0.f;
      x[4] = ov ? v.x : 0.f; x[5] = ov ? v.y : 0.f; x[6] = ov ? v.z : 0.f; x[7] = ov ? v.w : 0.f;
    } else {
      float raw[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) raw[e] = qa[(int64_t)(k + e < K ? k + e : 0) * s1];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = (rowok && k + e < K) ? raw[e] : 0.f;
    }
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_pair(x[2 * e], x[2 * e + 1], h[e], l[e]);
    char* dst = qf + ((int64_t)((kk * RT + tile) * 2) * 64 + lane) * 16;
    *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
    *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(l[0], l[1], l[2], l[3]);
  }
}

// r x r Gram-type products of Alg. 2 straight from the fragment images: a lane's 16 bytes of an image hold 8
// consecutive k of one row, which is the A-operand layout for rows of X and equally the B-operand layout for columns
// of S^T.  One workgroup (8 waves) per pair of products that share an image: X S^T and S S^T, i.e. (R' R^T, R R^T)
// with X = R', S = R and ((L^T L')^T, L^T L) with X = L'^T, S = L^T.  The two images are copied global -> LDS
// without registers, in halves of a 64-column chunk through a ring of four buffers per image, so that every image
// byte is read from L2 once per pair (read per wave, or once per product, the launch was bound by L2 bandwidth);
// wave w owns column tile w % 4 of both results (all row tiles) and k-step w / 4 of every half.  In the first GD
// iteration X = S and one product serves both outputs.  A long contraction is cut into segments, one workgroup each
// (chunks c0 .. c1 - 1): a segment leaves its partial sums for gram_finish_kernel.
template <int RT>
__device__ __forceinline__ void gram_emit(const float* Mss, const float* Mxs, const Bases& bs, int64_t off_out_ss,
                                          int64_t off_out_xs, int64_t off_img_ss, int64_t off_img_xs, int r,
                                          int transpose_xs, int nthreads);

template <int RT>
__device__ __forceinline__ void gram_body(const GramItem& it, const Bases& bs, unsigned char* smem) {
  constexpr int R = 32 * RT;
  constexpr int QF = qf_chunk_bytes(R);
  const int lane = threadIdx.x & 63, l32 = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cw = wave & 3, kh = wave >> 2;                            // column tile of the results; half of the k-steps of a chunk
  const char* __restrict__ X = bs.ws + it.off_x;
  const char* __restrict__ S = bs.ws + it.off_s;
  const bool same = it.off_x == it.off_s;
  // this workgroup's chunks (the images are zero-padded to whole chunks), walked in halves of 32 columns: a ring of
  // four half-chunk buffers per image keeps two to three copies in flight while one half is multiplied
  constexpr int HB = QF / 2;                                          // bytes of half a chunk of one image
  constexpr int NP = HB / 1024;                                       // 1 KB pieces of half a chunk: one copy instruction each
  constexpr int LPC = NP >= 8 ? NP / 8 : 1;                           // copy instructions per wave, image and half (waves beyond NP issue none)
  const int h_first = 2 * it.c0, h_end = 2 * it.c1;
  lds_u8* const lds = (lds_u8*)smem;                                  // [4 buffers][S | X][HB]
  auto copy = [&](int h, int buf) {
#pragma unroll
    for (int u = 0; u < LPC; ++u) {
      const int k = wave + 8 * u;
      if (k >= NP) continue;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(S + (int64_t)h * HB + k * 1024 + lane * 16),
                                       (__attribute__((address_space(3))) void*)(lds + (buf * 2) * HB + k * 1024), 16, 0, 0);
      if (!same)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(X + (int64_t)h * HB + k * 1024 + lane * 16),
                                         (__attribute__((address_space(3))) void*)(lds + (buf * 2 + 1) * HB + k * 1024), 16, 0, 0);
    }
  };
  f32x16 ass[RT], axs[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) ass[t][i] = axs[t][i] = 0.f;
  for (int h = h_first; h < h_end && h < h_first + 3; ++h) copy(h, h & 3);
  for (int h = h_first; h < h_end; ++h) {
    // half h has landed: every wave waits until at most the copies it issued after h are in flight (LPC instructions
    // per copy, twice that with two images), the barrier collects the waves and says that everybody is done with
    // half h - 1, whose buffer half h + 3 goes to
    const int newer = h_end - 1 - h < 2 ? h_end - 1 - h : 2;
    if (newer == 2) {
      if (same) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPC) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(4 * LPC) : "memory");
    } else if (newer == 1) {
      if (same) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPC) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPC) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    wg_barrier();
    if (h + 3 < h_end) copy(h + 3, (h + 3) & 3);
    if (cw < RT) {
      const unsigned ss = lds_addr(lds) + ((h & 3) * 2) * HB, xs = ss + HB;
      const int kk = kh;                                              // a half holds two 16-wide k-steps: one per wave half
      bf16x8 ah[RT], al[RT];
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        ah[t] = lds_frag_raw(ss + (((kk * RT + t) * 2) * 64 + lane) * 16);
        al[t] = lds_frag_raw(ss + (((kk * RT + t) * 2 + 1) * 64 + lane) * 16);
      }
      bf16x8 bh = lds_frag_raw(ss + (((kk * RT + cw) * 2) * 64 + lane) * 16);
      bf16x8 bl = lds_frag_raw(ss + (((kk * RT + cw) * 2 + 1) * 64 + lane) * 16);
#pragma unroll
      for (int t = 0; t < RT; ++t) lds_wait(ah[t], al[t], bh, bl);
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        ass[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[t], bh, ass[t], 0, 0, 0);
        ass[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[t], bh, ass[t], 0, 0, 0);
        ass[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[t], bl, ass[t], 0, 0, 0);
      }
      if (!same) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          ah[t] = lds_frag_raw(xs + (((kk * RT + t) * 2) * 64 + lane) * 16);
          al[t] = lds_frag_raw(xs + (((kk * RT + t) * 2 + 1) * 64 + lane) * 16);
        }
#pragma unroll
        for (int t = 0; t < RT; ++t) lds_wait(ah[t], al[t], bh, bl);
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          axs[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[t], bh, axs[t], 0, 0, 0);
          axs[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[t], bh, axs[t], 0, 0, 0);
          axs[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[t], bl, axs[t], 0, 0, 0);
        }
      }
    }
  }
  // the two halves of the k-steps are added through LDS (the image buffers are free now), in a fixed order
  __syncthreads();
  float* part = reinterpret_cast<float*>(smem) + (cw * RT * 16) * 64;  // [product][column tile][row tile][16][lane]
  float* part2 = part + 4 * RT * 16 * 64;
  if (kh == 1 && cw < RT) {
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        part[(t * 16 + i) * 64 + lane] = ass[t][i];
        if (!same) part2[(t * 16 + i) * 64 + lane] = axs[t][i];
      }
  }
  __syncthreads();
  const bool owner = kh == 0 && cw < RT;
  if (owner) {
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        ass[t][i] += part[(t * 16 + i) * 64 + lane];
        axs[t][i] = same ? ass[t][i] : axs[t][i] + part2[(t * 16 + i) * 64 + lane];
      }
  }
  __syncthreads();                                                     // the partial sums are read: LDS takes the results
  float* const Mss = reinterpret_cast<float*>(smem);                   // [R][R] each; rows and columns beyond r are zero
  float* const Mxs = Mss + R * R;                                      // (the images of the factors are zero-padded)
  if (it.nseg > 1) {
    // one segment of a long contraction: leave the two partial matrices for gram_finish_kernel
    if (owner) {
      float* __restrict__ part_ss = reinterpret_cast<float*>(bs.ws + it.off_part) + (int64_t)it.seg * 2 * R * R;
      float* __restrict__ part_xs = part_ss + R * R;
      const int col = 32 * cw + l32;
#pragma unroll
      for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int row = 32 * t + 8 * q + 4 * lh + p;
            part_ss[row * R + col] = ass[t][4 * q + p];
            if (!same) part_xs[row * R + col] = axs[t][4 * q + p];
          }
    }
    return;
  }
  if (owner) {
    const int col = 32 * cw + l32;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int row = 32 * t + 8 * q + 4 * lh + p;
          Mss[row * R + col] = ass[t][4 * q + p];
          Mxs[row * R + col] = axs[t][4 * q + p];
        }
  }
  __syncthreads();
  gram_emit<RT>(Mss, Mxs, bs, it.off_out_ss, it.off_out_xs, it.off_img_ss, it.off_img_xs, it.r, it.transpose_xs, 512);
}

// Results of a pair of Gram-type products, complete in LDS as [R][R] fp32 each: the r x r matrices themselves and
// their fragment images for the GD step on the stripes (the layout qf_image_kernel writes), 64-wide chunks of the
// contraction index k: lane l of a piece holds result[64 c + 16 kk + 8 (l / 32) .. + 7][32 tile + l % 32].
template <int RT>
__device__ __forceinline__ void gram_emit(const float* Mss, const float* Mxs, const Bases& bs, int64_t off_out_ss,
                                          int64_t off_out_xs, int64_t off_img_ss, int64_t off_img_xs, int r,
                                          int transpose_xs, int nthreads) {
  constexpr int R = 32 * RT;
  constexpr int QF = qf_chunk_bytes(R);
  float* __restrict__ Oss = reinterpret_cast<float*>(bs.ws + off_out_ss);
  float* __restrict__ Oxs = reinterpret_cast<float*>(bs.ws + off_out_xs);
  for (int id = threadIdx.x; id < r * r; id += nthreads) {
    const int row = id / r, col = id % r;
    Oss[id] = Mss[row * R + col];
    Oxs[id] = transpose_xs ? Mxs[col * R + row] : Mxs[row * R + col];      // the transposition is an LDS read: stores stay contiguous
  }
  if (off_img_ss < 0) return;
  const int nk2 = (r + BK - 1) / BK;
  for (int p = threadIdx.x; p < 2 * nk2 * (BK / 16) * RT * 64; p += nthreads) {
    const int ln = p & 63, rest = p >> 6, tile = rest % RT, kk = (rest / RT) % (BK / 16), kc = (rest / (RT * (BK / 16))) % nk2;
    const int which = rest / (RT * (BK / 16) * nk2);
    const float* M = (which ? Mxs : Mss) + 32 * tile + (ln & 31);
    const int k0 = BK * kc + 16 * kk + 8 * (ln >> 5);
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = k0 + e < R ? M[(k0 + e) * R] : 0.f;
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) split_pair(x[2 * e], x[2 * e + 1], h[e], l[e]);
    char* dst = bs.ws + (which ? off_img_xs : off_img_ss) + (int64_t)kc * QF + ((int64_t)((kk * RT + tile) * 2) * 64 + ln) * 16;
    *reinterpret_cast<uint4*>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
    *reinterpret_cast<uint4*>(dst + 1024) = make_uint4(l[0], l[1], l[2], l[3]);
  }
}

__global__ __launch_bounds__(512) void gram_kernel(const GramItem* __restrict__ items, Bases bs) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * qf_chunk_bytes(128)];
  const GramItem it = items[blockIdx.x];
  if (it.rc == 32) gram_body<1>(it, bs, smem);
  else if (it.rc == 64) gram_body<2>(it, bs, smem);
  else gram_body<4>(it, bs, smem);
}

// Sum of the partial results that the segments of a long contraction left (fixed order: segment 0, 1, ...), then the
// same results and images a single-segment workgroup writes itself.
template <int RT>
__device__ __forceinline__ void gram_finish_body(const GramFinItem& it, const Bases& bs, unsigned char* smem) {
  constexpr int R = 32 * RT;
  float* const Mss = reinterpret_cast<float*>(smem);
  float* const Mxs = Mss + R * R;
  // 16 bytes per load, every load of a thread independent of the others: the launch is a few latencies long
  const float4* __restrict__ part = reinterpret_cast<const float4*>(bs.ws + it.off_part);
  constexpr int Q = R * R / 4;                       // float4 per matrix
  constexpr int PER = (Q + 511) / 512;               // per thread: 8 at R = 128
  float4 a[PER], x[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) a[u] = x[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sg = 0; sg < it.nseg; ++sg) {
    float4 pa[PER], px[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int id = threadIdx.x + 512 * u;
      if (id < Q) {
        pa[u] = part[(int64_t)sg * 2 * Q + id];
        if (!it.same) px[u] = part[(int64_t)sg * 2 * Q + Q + id];
      }
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int id = threadIdx.x + 512 * u;
      if (id < Q) {
        a[u].x += pa[u].x; a[u].y += pa[u].y; a[u].z += pa[u].z; a[u].w += pa[u].w;
        if (!it.same) { x[u].x += px[u].x; x[u].y += px[u].y; x[u].z += px[u].z; x[u].w += px[u].w; }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int id = threadIdx.x + 512 * u;
    if (id < Q) {
      reinterpret_cast<float4*>(Mss)[id] = a[u];
      reinterpret_cast<float4*>(Mxs)[id] = it.same ? a[u] : x[u];
    }
  }
  __syncthreads();
  gram_emit<RT>(Mss, Mxs, bs, it.off_out_ss, it.off_out_xs, it.off_img_ss, it.off_img_xs, it.r, it.transpose_xs, 512);
}

__global__ __launch_bounds__(512) void gram_finish_kernel(const GramFinItem* __restrict__ items, Bases bs) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * 128 * 128 * 4];
  const GramFinItem it = items[blockIdx.x];
  if (it.rc == 32) gram_finish_body<1>(it, bs, smem);
  else if (it.rc == 64) gram_finish_body<2>(it, bs, smem);
  else gram_finish_body<4>(it, bs, smem);
}

template <int RT>
void launch_proj_rt(bool w16, bool vel, dim3 grid, const ProjItem* items, const LrBlockDev* lrb, Bases b, StepScalars sc,
                    hipStream_t s) {
  if (w16 && vel) hipLaunchKernelGGL((proj_kernel<RT, true, true>), grid, dim3(NT), 0, s, items, lrb, b, sc);
  else if (w16) hipLaunchKernelGGL((proj_kernel<RT, true, false>), grid, dim3(NT), 0, s, items, lrb, b, sc);
  else if (vel) hipLaunchKernelGGL((proj_kernel<RT, false, true>), grid, dim3(NT), 0, s, items, lrb, b, sc);
  else hipLaunchKernelGGL((proj_kernel<RT, false, false>), grid, dim3(NT), 0, s, items, lrb, b, sc);
}

}  // namespace

size_t proj_qf_bytes(int r, int n) { return (size_t)((n + BK - 1) / BK) * qf_chunk_bytes(r); }
size_t proj_timg_bytes(int r, int n) { return (size_t)((n + BK - 1) / BK) * timg_chunk_bytes(r); }

// vel: every block of the list keeps a per-element second moment (v_kind 0); otherwise none does
void launch_proj(int rt, bool w16, bool vel, const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b,
                 StepScalars sc, hipStream_t s) {
  if (nitems <= 0) return;
  const dim3 grid((unsigned)nitems);
  if (rt == 1) launch_proj_rt<1>(w16, vel, grid, items, lrb, b, sc, s);
  else if (rt == 2) launch_proj_rt<2>(w16, vel, grid, items, lrb, b, sc, s);
  else launch_proj_rt<4>(w16, vel, grid, items, lrb, b, sc, s);
}

void launch_stripe(int rt, bool tra, const StripeItem* items, int64_t nitems, const StripeProb* probs, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  const dim3 grid((unsigned)nitems);
  if (tra) {
    if (rt == 1) hipLaunchKernelGGL((stripe_kernel<1, true>), grid, dim3(NT), 0, s, items, probs, b);
    else if (rt == 2) hipLaunchKernelGGL((stripe_kernel<2, true>), grid, dim3(NT), 0, s, items, probs, b);
    else hipLaunchKernelGGL((stripe_kernel<4, true>), grid, dim3(NT), 0, s, items, probs, b);
  } else {
    if (rt == 1) hipLaunchKernelGGL((stripe_kernel<1, false>), grid, dim3(NT), 0, s, items, probs, b);
    else if (rt == 2) hipLaunchKernelGGL((stripe_kernel<2, false>), grid, dim3(NT), 0, s, items, probs, b);
    else hipLaunchKernelGGL((stripe_kernel<4, false>), grid, dim3(NT), 0, s, items, probs, b);
  }
}

void launch_gram(const GramItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(gram_kernel, dim3((unsigned)nitems), dim3(512), 0, s, items, b);
}

void launch_gram_finish(const GramFinItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(gram_finish_kernel, dim3((unsigned)nitems), dim3(512), 0, s, items, b);
}

void launch_qt_image(const ImgItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(qt_image_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

template <int RT>
void launch_ru_rt(bool w16, dim3 grid, const ProjItem* items, const RuBlockDev* blocks, Bases b, StepScalars sc, hipStream_t s) {
  if (w16) hipLaunchKernelGGL((refresh_update_kernel<RT, true>), grid, dim3(NT), 0, s, items, blocks, b, sc);
  else hipLaunchKernelGGL((refresh_update_kernel<RT, false>), grid, dim3(NT), 0, s, items, blocks, b, sc);
}

void launch_refresh_update(int rt, bool w16, const ProjItem* items, int64_t nitems, const RuBlockDev* blocks, Bases b,
                           StepScalars sc, hipStream_t s) {
  if (nitems <= 0) return;
  const dim3 grid((unsigned)nitems);
  if (rt == 1) launch_ru_rt<1>(w16, grid, items, blocks, b, sc, s);
  else if (rt == 2) launch_ru_rt<2>(w16, grid, items, blocks, b, sc, s);
  else launch_ru_rt<4>(w16, grid, items, blocks, b, sc, s);
}

void launch_qf_image(const ImgItem* items, int64_t nitems, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(qf_image_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, b);
}

void launch_qimage(const QsItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, hipStream_t s) {
  if (nitems <= 0) return;
  hipLaunchKernelGGL(qimage_kernel, dim3((unsigned)nitems), dim3(256), 0, s, items, lrb, b);
}

}  // namespace adapm
