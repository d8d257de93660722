// Internal structures shared by the host planner and the gfx950 kernels.
//
// The host turns the block table into a fixed list of launches at adapm_init();
// every launch carries a device-resident work list, so a step is a short walk over
// that list (the "multi-tensor block scheduler").  Buffers are named by
// (space, block, byte offset) and resolved on the device against the base pointers
// handed to adapm_step().
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adapm {

enum Space : int32_t { SP_STATE = 0, SP_WS = 1, SP_GRAD = 2, SP_PARAM = 3, SP_NONE = 4 };
enum DType : int32_t { DT_F32 = 0, DT_BF16 = 1, DT_F64 = 2 };
enum VMode : int32_t { VM_ELEMENT = 0, VM_ROWGROUP = 1, VM_WHOLE = 2 };
enum MMode : int32_t { MM_NONE = 0, MM_FULL = 1, MM_LOWRANK = 2 };

struct Ref {
  int32_t space;
  int32_t block;   // used by SP_GRAD / SP_PARAM
  int64_t off;     // bytes from the base
};

struct Bases {
  char* state;
  char* ws;
  const void* const* grads;   // device array of nblocks pointers
  void* const* params;        // device array of nblocks pointers
  const float* gscale;        // device scalar of the global gradient clipping (the method sees gscale * G); null = 1
};

// factor that the global gradient-norm clipping puts on every gradient of this step
__device__ __forceinline__ float grad_scale(const Bases& b) { return b.gscale ? *b.gscale : 1.f; }

// 16-byte vectors at the alignment of their elements: rows of G, W, R and v start wherever the number of
// columns puts them (the hardware serves global and buffer accesses at any byte alignment)
struct __attribute__((packed, aligned(2))) u32x4_a2 { uint32_t x, y, z, w; };
struct __attribute__((packed, aligned(4))) f32x4_a4 { float x, y, z, w; };

__device__ __forceinline__ char* resolve(const Ref& r, const Bases& b) {
  switch (r.space) {
    case SP_STATE: return b.state + r.off;
    case SP_WS: return b.ws + r.off;
    case SP_GRAD: return (char*)b.grads[r.block] + r.off;
    case SP_PARAM: return (char*)b.params[r.block] + r.off;
    default: return nullptr;
  }
}

// ---------------------------------------------------------------------------
// fp64-accumulate strided two-product GEMM
//   Out[i,j] = a1 * sum_k A1[i,k] B1[k,j] + a2 * sum_k A2[i,k] B2[k,j] + g * X[i,j] + d * Y[i,j]
// element (i,j) of a matrix lives at base + (i*s0 + j*s1) * sizeof(dtype)
// ---------------------------------------------------------------------------
struct Mat {
  Ref ref;
  int64_t s0, s1;
  int32_t dtype;
  int32_t pad;
};

struct GemmProblem {
  Mat A1, B1, A2, B2, X, Y, Out;
  int32_t M, N, K1, K2;
  double a1, a2, g, d;
  int32_t scale_g;   // 1: the (single) product has the gradient as an operand and takes the clipping factor
  int32_t tri;       // fp64 kernel: 1 = A1 is lower triangular, 2 = B1 is lower triangular (zero part of the contraction skipped)
  int64_t off_s;     // >= 0: workspace offset of a device scalar s (double); then Out = g X + s (a1 A1 B1 + a2 A2 B2 + d Y)
};

struct GemmTile {
  uint32_t prob;
  uint16_t ti, tj;   // 64 x 64 output tile coordinates
};

// ---------------------------------------------------------------------------
// element-wise update (Alg. 1 last line, eq. 5, per-element v) and v statistics
// ---------------------------------------------------------------------------
struct BlockDev {
  int64_t numel;
  int64_t group_elems;   // elements sharing one v (1 for per-element v)
  int64_t off_m;         // state byte offset of m (full momentum) or -1
  int64_t off_v;         // state byte offset of v
  int64_t off_C;         // workspace byte offset of the m x n low-rank term, or -1
  int32_t param_dtype, grad_dtype, mom_mode, v_mode;
  float lr_scale, wd;
};

struct EwItem {          // one workgroup: `count` elements from `start` of `block`
  int64_t start;
  int32_t block;
  int32_t count;
};

struct VsItem {          // one wavefront: sum of g^2 over [start, start+count)
  int64_t start;
  int64_t out;           // direct: group index; else index into the partial-sum array
  int32_t block;
  int32_t count;
  int32_t direct;        // 1: this piece is the whole group, finish v here
  int32_t pad;
};

struct VfItem {          // one thread: fold the partial sums of one group
  int64_t part0;
  int64_t group;
  int32_t block;
  int32_t nparts;
};

struct StepScalars {
  float beta1, beta2, eps, clip;
  float lr;
  float inv_debias_m, inv_debias_v;   // 1/(1-beta1^t), 1/(1-beta2^t) or 1
  float cG, cC;                       // low-rank blocks: m^c = cG * G + cC * C
  float dL, dP;                       // fused step with R held: D = dL * L_{t-1} + dP * (G Q^T)
};

// ---------------------------------------------------------------------------
// fused step with R held (k_proj_mfma.hip)
// ---------------------------------------------------------------------------
struct LrBlockDev {
  int32_t block;           // index into the gradient / parameter pointer tables
  int32_t m, n, r;         // r: the block's rank (any value up to 128)
  int64_t off_L, off_Q;    // state: L (m x r), Q = R (r x n), fp32
  int64_t off_v;           // state: v
  int64_t off_Qf;          // ws: Q as bf16 (hi, lo) MFMA fragments, per 64-column chunk
  int64_t off_Timg;        // ws: Q^T as bf16 (hi, lo) padded LDS images, per 64-column chunk
  int32_t v_kind;          // 0 per element; 1 groups of v_group_rows rows finished inside the 128-row stripe;
                           // 2 finished beforehand by the statistics kernel
  int32_t v_group_rows;
  int32_t param_dtype;
  float lr_scale, wd;
  int32_t rc;              // rank class the kernels are compiled for: 32, 64 or 128 >= r (images are zero-padded to it)
};

struct ProjItem {          // one workgroup: 128 rows of one block; lr < 0 = padding
  int32_t lr;
  int32_t row0;
};

struct QsItem {            // one workgroup: one 64-column chunk of Q
  int32_t lr;
  int32_t c;
};

// Stripe product of Alg. 2 (MFMA path): Out = A Q^T with A a bf16 matrix streamed once, Q (r x K, fp32)
// given as a bf16 (hi, lo) fragment image.  Used for G R^T (A = G) and for (L^T G)^T = G^T L (A = G^T, Q = L^T;
// what is stored is G, its column stripes are read transposed), whose result is written back transposed.
struct StripeProb {
  Ref a;                   // A: M x K bf16, row-major, row stride K; with transpose_out: A^T (K x M, row stride M) instead
  int32_t M, K, r;         // r: rows of Q actually present
  int32_t transpose_out;   // 0: Out is M x r (row stride r); 1: Out is r x M (row stride M)
  int32_t rc, upd;         // rank class of the image: 32, 64 or 128 >= r; upd: the factor update of Alg. 2 follows
  int64_t off_img;         // workspace: fragment image of Q
  int64_t off_out;         // workspace: fp32 result
  // upd != 0: Out = X + s (c1 X B1 + c2 X' B2 + cp A Q^T), the GD step of Alg. 2 on the factor X (X' = the factor of
  // the previous step), all three in the layout of Out; B1, B2 = r x r matrices given as fragment images of their
  // transposes (image row a, column k = B[k][a]); s = the double at workspace offset off_s (1 if off_s < 0)
  Ref x_cur, x_prev;
  int64_t off_b1, off_b2;
  int64_t off_s;
  int64_t off_next;        // >= 0: workspace offset where the fragment image of the new factor goes (its chunks run along M)
  int64_t off_timg;        // >= 0 (transposed output only): workspace offset where the image of the new factor's transpose
                           // goes ([hi|lo][column][R] per 64-column chunk, what the fused update reads)
  int64_t off_timg_prev;   // >= 0 (transposed output, first GD iteration only): the same image of the factor the iteration starts from
  float c1, c2, cp;
  // v_rows > 0 (A is the gradient itself): the blockwise second moment of the block is finished here,
  // v_g <- beta2 v_g + (1 - beta2) mean of g^2 over the v_rows rows of group g (state offset off_v, one float per group)
  float beta2;
  int64_t off_v;
  int32_t v_rows, pad2;
};
struct StripeItem {        // one workgroup: 128 rows of A; prob < 0 = padding
  int32_t prob;
  int32_t row0;
};
struct ImgItem {           // one workgroup: one 64-column chunk of the fragment image of Q(a, k) = q[a * s0 + k * s1]
  Mat q;                   // fp32
  int32_t r, K, c, rc;     // rows of Q, columns, chunk, rank class of the image (rows r .. rc-1 are zero)
  int64_t off_img;
};
struct GramItem {          // one workgroup: Out_xs = X S^T (stored transposed if transpose_xs) and Out_ss = S S^T, both r x r
  int64_t off_x, off_s;    // with row stride r, from the fragment images of X, S (r x K); workspace: images (rank class rc)
  int64_t off_out_xs, off_out_ss;   // workspace: fp32
  int64_t off_img_xs, off_img_ss;   // workspace: fragment images of the two results as the GD step on the stripes reads them
                                    // (image row a, column k = result[k][a]; S S^T is symmetric up to rounding); < 0: none
  int32_t K, r, rc, transpose_xs;
  // A long contraction is cut into segments of 64-column chunks, one workgroup each: segment [c0, c1) of nseg; with
  // nseg > 1 the workgroup only leaves its partial sums (two R x R fp32 matrices, S S^T then X S^T) at workspace
  // offset off_part + seg * 2 R^2 floats, and gram_finish_kernel adds them in segment order and writes the results.
  int32_t c0, c1, seg, nseg;
  int64_t off_part;
};
struct GramFinItem {       // one workgroup: the sum of the nseg partial results of one pair of products -> results and images
  int64_t off_part;
  int64_t off_out_xs, off_out_ss;
  int64_t off_img_xs, off_img_ss;
  int32_t r, rc, transpose_xs, nseg, same, pad;   // same: X = S (first GD iteration), one product serves both outputs
};
struct CopyItem {          // one workgroup: count floats from src + first to dst + first (first is a multiple of 4)
  Ref src, dst;
  int64_t first;
  int32_t count, pad;
};
constexpr int COPY_CHUNK = 16384;   // floats per workgroup
struct GrpItem {           // one workgroup of the grouped update: groups g0 .. g0 + ngroups - 1 of a block's blockwise v
  int64_t g0;
  int32_t block;
  int32_t ngroups;
};
constexpr int GRP_MAX_ELEMS = 2048;   // a wavefront holds one whole group of v in registers: 64 lanes x 4 vectors x 8
struct GnormItem {         // one workgroup: s = 1 / max(||A||_F, ||B||_F) for two r x r matrices (1 if both vanish)
  int64_t off_a, off_b;    // workspace
  int64_t off_out;         // workspace, one double
  int32_t r, dtype;        // DT_F32 or DT_F64
};

// Fused update of a step that ran Alg. 2 (MFMA path): m^c = cG G + cC (a1 L1 Q1 + a2 L2 Q2) tile by tile, never
// stored; (L1, Q1) = (L_{t-1}, R_{t-1}), (L2, Q2) = (L_t, R_t), (a1, a2) = (1, -1) with the bias correction of
// eq. 4 and (0, 1) without it.  Q1, Q2 are given as bf16 (hi, lo) images of their transposes.
struct RuBlockDev {
  int32_t block;           // index into the gradient / parameter pointer tables
  int32_t m, n, r, rc;     // rank and the rank class (32 / 64 / 128) of the kernel and the images
  int32_t v_kind;          // 0 per element (updated here); 2 finished beforehand, one value per v_group_rows rows
  int32_t v_group_rows;
  int32_t param_dtype;
  float lr_scale, wd, a1, a2;
  Ref l1, l2;              // fp32, m x r, row stride r
  Ref q1, q2;              // fp32, r x n, row stride n (read for a row's last n mod 8 columns only)
  int64_t off_img1, off_img2;   // workspace: images of Q1^T, Q2^T (layout of the held-R kernel's second image)
  int64_t off_v;           // state
};

struct SketchItem {      // seeded start R_0 of one low-rank block
  int64_t off_R;         // state byte offset
  int64_t count;         // rank * cols
  uint64_t key;
  float amp;
  int32_t pad;
};

// ---------------------------------------------------------------------------
// fp64 Cholesky + triangular inverse used by the orthonormalisation of R (T > 1)
// ---------------------------------------------------------------------------
struct CholItem {
  int64_t off_gram;      // ws: r x r fp64 Gram matrix R R^T, overwritten by its lower factor C (upper part zeroed)
  int64_t off_inv;       // ws: r x r fp64, receives C^-1 (lower triangular, upper part zeroed)
  int32_t r;
  int32_t pad;
};

// In-place re-expression of the factors after the Cholesky factorisation (T > 1, MFMA path): one workgroup owns 64
// whole columns of R (R <- C^-1 R) or 64 whole rows of L (L <- L C), so nothing it overwrites is read by another.
struct RegaugeItem {
  int64_t off_x;         // state: the factor (fp32), R (r x len, row stride len) or L (len x r, row stride r)
  int64_t off_c;         // ws: C^-1 (for R) or C (for L), r x r fp64, lower triangular
  int32_t r, len;        // rank; columns of R / rows of L
  int32_t first;         // first column / row of this workgroup's 64
  int32_t is_L;
};

// launchers (defined next to their kernels)
void launch_gemm64(const GemmProblem* probs, const GemmTile* tiles, int64_t ntiles, Bases b, hipStream_t s);
void launch_vstat(const BlockDev* blocks, const VsItem* items, int64_t nitems, double* partials, Bases b,
                  float beta2, hipStream_t s);
void launch_vfinal(const BlockDev* blocks, const VfItem* items, int64_t nitems, const double* partials, Bases b,
                   float beta2, hipStream_t s);
void launch_gram_norm(const GnormItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_update_grouped(const BlockDev* blocks, const GrpItem* items, int64_t nitems, Bases b, StepScalars sc,
                           hipStream_t s);
void launch_gradnorm_final(const double* partials, int64_t nparts, float max_norm, float* out, hipStream_t s);
void launch_update(const BlockDev* blocks, const EwItem* items, int64_t nitems, Bases b, StepScalars sc,
                   hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);
void launch_copy(const CopyItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_sketch(const SketchItem* items, int64_t nitems, char* state, hipStream_t s);
void launch_chol(const CholItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_regauge_apply(const RegaugeItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_gemm_mfma(const GemmProblem* probs, const GemmTile* tiles, int64_t ntiles, Bases b, hipStream_t s);
void launch_proj(int rt, bool w16, bool vel, const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b,
                 StepScalars sc, hipStream_t s);
// the same step for rank class 128, bf16 parameters, blockwise v, columns % 8 == 0 and <= proj_keep_max_cols():
// stripes of proj_keep_rows() rows whose gradient stays on chip between the two passes (k_proj_keep.hip)
void launch_proj_keep(const ProjItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, StepScalars sc, hipStream_t s);
int proj_keep_rows();
int proj_keep_max_cols();
void launch_qimage(const QsItem* items, int64_t nitems, const LrBlockDev* lrb, Bases b, hipStream_t s);
void launch_stripe(int rt, bool tra, const StripeItem* items, int64_t nitems, const StripeProb* probs, Bases b, hipStream_t s);
void launch_qf_image(const ImgItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_gram(const GramItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_gram_finish(const GramFinItem* items, int64_t nitems, Bases b, hipStream_t s);
constexpr int GRAM_SEG_CHUNKS = 25;    // shortest segment of a Gram-type product in 64-column chunks (1600 columns): sizes the partial sums
void launch_qt_image(const ImgItem* items, int64_t nitems, Bases b, hipStream_t s);
void launch_refresh_update(int rt, bool w16, const ProjItem* items, int64_t nitems, const RuBlockDev* blocks, Bases b,
                           StepScalars sc, hipStream_t s);
size_t proj_qf_bytes(int r, int n);     // sizes of the two images of Q kept for the fused step
size_t proj_timg_bytes(int r, int n);

}  // namespace adapm
