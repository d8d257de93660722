// Host side of the AdaPM step library: table validation, state / workspace layout,
// the launch plan ("multi-tensor block scheduler") and the C ABI of include/adapm.h.
//
// adapm_init() walks the block table once and emits, for every phase of a step, one
// device-resident work list covering all blocks; adapm_step() then enqueues a short,
// fixed sequence of launches on the caller's stream.  Nothing here computes any part of
// the update on the host.
#include "../../include/adapm.h"
#include "adapm_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

using namespace adapm;

namespace {

thread_local std::string g_err;

adapm_status_t fail(adapm_status_t code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) return fail(ADAPM_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr size_t ALIGN = 256;
size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

constexpr int EW_CHUNK = 8192;      // elements per workgroup of the update kernel
constexpr int VS_CHUNK = 16384;     // elements per wavefront of the v-statistics kernel

enum Path { PATH_NONE = 0, PATH_F64 = 1, PATH_FAST = 2 };

struct Layout {                      // byte offsets, -1 = absent
  int64_t sL = -1, sR = -1, sm = -1, sv = -1;               // state
  int64_t wLa = -1, wRa = -1, wLb = -1, wRb = -1;           // ws: ping-pong factors of Alg. 2
  int64_t wP = -1, wS = -1, wGrr = -1, wGpr = -1, wGll = -1, wGlp = -1;
  int64_t wG64 = -1, wCinv = -1, wC = -1;
  int64_t wQf = -1, wTimg = -1;                             // ws: bf16 (hi, lo) images of Q and Q^T
  int64_t wIr = -1, wIl = -1;                               // ws: the fragment images of R, L^T during Alg. 2 ...
  int64_t wIr2 = -1, wIl2 = -1;                             // ws: ... written by the stripes of one GD iteration for the next, hence two sets
  int64_t wIr0 = -1, wIl0 = -1;                             // ws: the same images of R_{t-1}, L_{t-1}^T (first iteration; Gram matrices)
  int64_t wGpn = -1, wGpm = -1;                             // ws: partial sums of the Gram-type products over n and over m, where those are cut into segments
  int64_t wNu = -1;                                         // ws: normaliser of the optional scale-normalised Alg. 2 (one double)
  int64_t wB[4] = {-1, -1, -1, -1};                         // ws: fragment images of R R^T, R' R^T, L^T L, L^T L' (transposed as the fused GD step needs them)
  int64_t wT1 = -1, wT2 = -1;                               // ws: images of R_{t-1}^T and R_t^T for the fused update after Alg. 2
  int64_t nv = 0;
  int path = PATH_NONE;
};

enum OpKind { OP_GEMM, OP_GEMM_MFMA, OP_CHOL, OP_VSTAT, OP_VFINAL, OP_UPDATE, OP_QSPLIT, OP_PROJ, OP_QFIMG, OP_STRIPE, OP_QTIMG, OP_REFRESH_UPDATE, OP_GRADNORM, OP_GRAM, OP_GNORM, OP_UPDATE_GROUPED, OP_COPY, OP_PROJ_KEEP, OP_GRAM_FIN, OP_REGAUGE_APPLY };

struct GemmList {
  std::vector<GemmProblem> probs;
  std::vector<GemmTile> tiles;
  GemmProblem* d_probs = nullptr;
  GemmTile* d_tiles = nullptr;
  int tile = 64;
};

struct Op {
  OpKind kind;
  int index;          // GEMM*: gemm list; UPDATE / VSTAT / VFINAL / PROJ / QFIMG / STRIPE / ...: which item list
  float cG, cC;       // UPDATE of low-rank blocks, PROJ
  const char* label;  // profiling name
  int aux = 0;        // REFRESH_UPDATE: which list of block descriptors the items index
};

template <class T>
struct DevList {
  std::vector<T> h;
  T* d = nullptr;
};

Mat mat(int32_t space, int32_t block, int64_t off, int64_t s0, int64_t s1, int32_t dtype) {
  Mat m;
  m.ref = Ref{space, block, off};
  m.s0 = s0; m.s1 = s1; m.dtype = dtype; m.pad = 0;
  return m;
}
Mat none_mat() { return mat(SP_NONE, 0, 0, 0, 0, DT_F32); }

struct ProfRec {
  const char* label;
  hipEvent_t e0, e1;
};

}  // namespace

struct adapm_ctx {
  std::vector<adapm_block_t> table;
  adapm_hparams_t hp;
  std::vector<Layout> lay;
  size_t state_bytes = 0, ws_bytes = 0;
  int64_t off_partials = -1;
  int64_t off_gn_partials = -1, off_gn_out = -1;   // ws: global gradient norm (partial sums; norm and factor)
  float grad_clip = 0.f;                           // threshold of the global gradient-norm clipping; <= 0: off

  DevList<BlockDev> blocks;
  std::vector<DevList<EwItem>> ew;   // 0: full / no momentum; then one per group of low-rank blocks on the F64 path (the MFMA path updates in its fused kernels)
  DevList<VsItem> vs[2];        // 0: every step; 1: only on steps that run Alg. 2 (fused elsewhere)
  DevList<VfItem> vf[2];
  DevList<GrpItem> grp;         // full / no momentum blocks whose v groups fit a wavefront: statistic + update fused
  DevList<VsItem> gn;           // every gradient in pieces: sums of squares for the global norm
  DevList<SketchItem> sk;
  std::vector<DevList<CholItem>> chol;   // per group of low-rank blocks (T > 1)
  DevList<LrBlockDev> lrb;
  DevList<ProjItem> proj[12];   // (rank 32 / 64 / 128) x (fp32 / bf16 parameters) x (blockwise / per-element v)
  DevList<ProjItem> proj_keep;  // rank class 128, bf16 parameters, blockwise v, short rows: 64-row stripes whose G stays on chip
  DevList<QsItem> qs;
  DevList<StripeProb> sprob;            //   stripe products G R^T and G^T L ...
  std::vector<DevList<ImgItem>> img;    //   ... per GD iteration: fragment images of R and L^T (only the first iteration has any: the stripes write the later ones)
  std::vector<DevList<StripeItem>> sit; //   ... per GD iteration x rank class: the stripes
  std::vector<DevList<GramFinItem>> gfin; //   ... same index as gram: the sums over the segments of the long ones
  std::vector<DevList<GramItem>> gram;  //   ... per GD iteration: the four r x r Gram-type products, from the images, in pairs that share one
  std::vector<DevList<GnormItem>> gnorm; // optional scale-normalised Alg. 2: per (path, GD iteration) the normalisers
  // per group of low-rank blocks (a group runs Alg. 2 from start to end in one region of scratch, see build_plan):
  std::vector<DevList<CopyItem>> cp;    // T = 1, MFMA path: the factors Alg. 2 leaves in the workspace -> state
  std::vector<DevList<RuBlockDev>> rub; // fused update after Alg. 2 (MFMA path): blocks, images of R^T, stripes
  std::vector<DevList<ImgItem>> qt;
  std::vector<DevList<ProjItem>> ru;    //   6 per group: (rank class 32 / 64 / 128) x (fp32 / bf16 parameters)
  int n_groups = 0;
  int rg_gram = -1, rg_chol = -1;       // T > 1, MFMA path: the re-expression of all blocks' factors after the last group
  DevList<RegaugeItem> rg_apply;
  std::vector<GemmList> gemms;
  std::vector<Op> seq_refresh, seq_project;

  bool uploaded = false;
  int device = -1;
  char* arena = nullptr;
  // Pointer tables ([2 * nblocks]: params then grads) live on the device in a few slots, each with a pinned host
  // copy.  A step whose pointers equal a slot's reuses it (no copy: a caller that rotates two or three sets of
  // gradient tensors uploads each set once); otherwise the least recently used slot is rewritten by a copy on the
  // step's stream.  Its pinned copy may only be overwritten once the copy that last read it has finished: that is
  // asked of the slot's event without blocking, and waited for only in the (pathological) case that a copy issued
  // NSLOT - 1 uploads ago is still pending.
  static constexpr int NSLOT = 4;
  struct PtrSlot {
    void** d = nullptr;
    void** h = nullptr;
    hipEvent_t copied = nullptr;
    bool valid = false;
    uint64_t last_use = 0;
  } slot[NSLOT];
  uint64_t use_clock = 0;
  bool keep_enabled = false;            // ADAPM_PROJ_KEEP=1 in the environment at adapm_init: blocks that qualify run in the kernel
                                        // that keeps G on chip between the passes (one read of G; measured slower than the two-read
                                        // kernel on MI355X, so it is off by default and kept for the comparison)
  bool gauge_ok = false;                // T > 1: the state's R has orthonormal rows (a step that ran Alg. 2, or adapm_state_loaded)
  int64_t last_launches = 0;
  int n_lowrank = 0;
  const void* split_ws = nullptr;       // workspace that holds valid bf16 copies of Q (T > 1, MFMA path) ...
  const void* split_state = nullptr;    // ... made from the R of this state buffer
  std::vector<std::pair<std::string, std::pair<double, int64_t>>> prof_agg;   // folded timings (adapm_profile_read)

  bool profiling = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> event_pool;
};

namespace {

int64_t num_v(const adapm_block_t& b) {
  if (b.v_mode == ADAPM_V_ELEMENT) return b.rows * b.cols;
  if (b.v_mode == ADAPM_V_ROWGROUP) return b.rows / b.v_group_rows;
  return 1;
}
int64_t group_elems(const adapm_block_t& b) {
  if (b.v_mode == ADAPM_V_ELEMENT) return 1;
  if (b.v_mode == ADAPM_V_ROWGROUP) return (int64_t)b.v_group_rows * b.cols;
  return b.rows * b.cols;
}
int esize(int32_t dt) { return dt == ADAPM_BF16 ? 2 : 4; }

// BF16X2 needs bf16 gradients and a rank of at most 128; other blocks use F64.  The number of columns is free:
// the fused kernels read 8-element vectors at whatever alignment the rows have and finish a row's last
// cols mod 8 columns element by element.
// rank class the MFMA kernels are compiled for (the bf16 images of the factors are zero-padded to it); 0 = none
int rank_class(int r) { return r <= 32 ? 32 : (r <= 64 ? 64 : (r <= 128 ? 128 : 0)); }

int path_of(const adapm_block_t& b, const adapm_hparams_t& hp) {
  if (b.mom_mode != ADAPM_MOM_LOWRANK) return PATH_NONE;
  const bool want = hp.contraction == ADAPM_CONTRACT_BF16X2 ||
                    (hp.contraction == ADAPM_CONTRACT_AUTO && b.param_dtype == ADAPM_BF16);
  const bool can = b.grad_dtype == ADAPM_BF16 && rank_class(b.rank) != 0 && b.cols >= 8 &&
                   b.cols <= (1 << 21);   // 128 rows of a stripe stay inside one 32-bit buffer range
  return (want && can) ? PATH_FAST : PATH_F64;
}
// Alg. 2 on the MFMA path: the two products that stream G (G R^T and L^T G) run as stripe products when the rows
// of G are whole 16-byte vectors (both read G itself: stripes of rows, and stripes of columns in chunks of 64 rows)
bool stripe_ok(const adapm_block_t& b) { return b.cols % 8 == 0; }
// v of a block on the MFMA path can be finished inside the 128-row stripe of the fused kernel
bool v_fusable(const adapm_block_t& b) {
  return b.v_mode == ADAPM_V_ROWGROUP && b.v_group_rows <= 128 && 128 % b.v_group_rows == 0;
}

adapm_status_t validate(const adapm_block_t* t, int64_t n, const adapm_hparams_t* hp) {
  if (!t || !hp) return fail(ADAPM_EINVAL, "null table or hparams");
  if (n <= 0 || n > (1 << 24)) return fail(ADAPM_EINVAL, "nblocks %lld out of range", (long long)n);
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(ADAPM_EINVAL, "beta1/beta2 must lie in [0,1)");
  if (!(hp->eps >= 0.f) || !(hp->clip > 0.f)) return fail(ADAPM_EINVAL, "eps must be >= 0 and clip > 0");
  if (hp->refresh_iters_K < 1 || hp->refresh_iters_K > 1024) return fail(ADAPM_EINVAL, "refresh_iters_K out of range");
  if (hp->refresh_period_T < 1) return fail(ADAPM_EINVAL, "refresh_period_T must be >= 1");
  // the literal zero start never leaves zero (both gradients of Alg. 2 vanish there), and R = 0 has no orthonormal
  // re-expression: the step with R held is undefined for it
  if (hp->seed == 0 && hp->refresh_period_T > 1)
    return fail(ADAPM_EINVAL, "seed = 0 (the all-zero start of Alg. 1) needs refresh_period_T = 1");
  if (hp->adam_debias != 0 && hp->adam_debias != 1) return fail(ADAPM_EINVAL, "adam_debias must be 0 or 1");
  if (hp->bias_correction != 0 && hp->bias_correction != 1) return fail(ADAPM_EINVAL, "bias_correction must be 0 or 1");
  if (hp->refresh_normalise != 0 && hp->refresh_normalise != 1) return fail(ADAPM_EINVAL, "refresh_normalise must be 0 or 1");
  if (hp->contraction < ADAPM_CONTRACT_AUTO || hp->contraction > ADAPM_CONTRACT_BF16X2)
    return fail(ADAPM_EINVAL, "unknown contraction mode %d", hp->contraction);
  for (int64_t i = 0; i < n; ++i) {
    const adapm_block_t& b = t[i];
    if (b.rows < 1 || b.cols < 1) return fail(ADAPM_EINVAL, "block %lld: rows/cols must be >= 1", (long long)i);
    if (b.rows > (1ll << 31) || b.cols > (1ll << 31) || b.rows * b.cols >= (1ll << 40))
      return fail(ADAPM_EINVAL, "block %lld: too large", (long long)i);
    if ((b.param_dtype != ADAPM_F32 && b.param_dtype != ADAPM_BF16) ||
        (b.grad_dtype != ADAPM_F32 && b.grad_dtype != ADAPM_BF16))
      return fail(ADAPM_EINVAL, "block %lld: unknown dtype", (long long)i);
    if (b.mom_mode < ADAPM_MOM_NONE || b.mom_mode > ADAPM_MOM_LOWRANK)
      return fail(ADAPM_EINVAL, "block %lld: unknown mom_mode %d", (long long)i, b.mom_mode);
    if (b.mom_mode == ADAPM_MOM_LOWRANK) {
      if (b.cols < 2 || b.rows < 2) return fail(ADAPM_EINVAL, "block %lld: low-rank momentum needs a matrix", (long long)i);
      if (b.rank < 1 || b.rank > b.rows || b.rank > b.cols)
        return fail(ADAPM_EINVAL, "block %lld: rank %d not in [1, min(rows, cols)]", (long long)i, b.rank);
      if (b.rows >= (1ll << 22) || b.cols >= (1ll << 22))
        return fail(ADAPM_EINVAL, "block %lld: low-rank blocks are limited to 2^22 rows/cols", (long long)i);
    }
    if (b.v_mode < ADAPM_V_ELEMENT || b.v_mode > ADAPM_V_WHOLE)
      return fail(ADAPM_EINVAL, "block %lld: unknown v_mode %d", (long long)i, b.v_mode);
    if (b.v_mode == ADAPM_V_ROWGROUP && (b.v_group_rows < 1 || b.rows % b.v_group_rows != 0))
      return fail(ADAPM_EINVAL, "block %lld: rows %% v_group_rows != 0", (long long)i);
    if (!std::isfinite(b.lr_scale) || !std::isfinite(b.weight_decay))
      return fail(ADAPM_EINVAL, "block %lld: lr_scale / weight_decay not finite", (long long)i);
    if (hp->contraction == ADAPM_CONTRACT_BF16X2 && b.mom_mode == ADAPM_MOM_LOWRANK && b.grad_dtype != ADAPM_BF16)
      return fail(ADAPM_EINVAL, "block %lld: BF16X2 contraction needs bf16 gradients", (long long)i);
  }
  return ADAPM_OK;
}

uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// output tile edge: 64 for the fp64 kernel, 128 for the MFMA kernel
// lower_only: a symmetric result of which only the tiles on and below the diagonal are read afterwards
void add_problem(GemmList& gl, const GemmProblem& p, int tile = 0, bool lower_only = false) {
  if (tile) gl.tile = tile;
  gl.probs.push_back(p);
  const uint32_t id = (uint32_t)gl.probs.size() - 1;
  const int T = gl.tile;
  for (int ti = 0; ti < (p.M + T - 1) / T; ++ti)
    for (int tj = 0; tj < (p.N + T - 1) / T; ++tj)
      if (!lower_only || tj <= ti) gl.tiles.push_back(GemmTile{id, (uint16_t)ti, (uint16_t)tj});
}

GemmProblem problem(int M, int N) {
  GemmProblem p;
  memset(&p, 0, sizeof p);
  p.A1 = p.B1 = p.A2 = p.B2 = p.X = p.Y = p.Out = none_mat();
  p.M = M; p.N = N;
  p.off_s = -1;
  return p;
}

// most segments a Gram-type product over K columns is cut into (sizes the partial sums; a group may use fewer, longer ones)
int gram_segments(int64_t K) {
  const int64_t nch = (K + 63) / 64;
  return (int)((nch + GRAM_SEG_CHUNKS - 1) / GRAM_SEG_CHUNKS);
}

std::vector<double> effective_step_sizes(int K) {
  // App. B: eta_k = 0.5 (1 + cos(pi k / K)), k = 1..K.  A zero step changes nothing and is skipped.
  std::vector<double> out;
  for (int k = 1; k <= K; ++k) {
    const double eta = 0.5 * (1.0 + std::cos(M_PI * (double)k / (double)K));
    if (eta != 0.0) out.push_back(eta);
  }
  return out;
}

// Alg. 2 + eq. 3-4 for the low-rank blocks of one contraction path, as batched GEMM launches.
//   fast = false: fp64 vector-ALU GEMM, every intermediate kept in fp64;
//   fast = true : split-bf16 MFMA GEMM, fp32 intermediates.
// `ids`: the blocks of ONE group, all on the same contraction path; the group's scratch offsets are in c->lay.
void plan_lowrank_refresh(adapm_ctx* c, bool fast, const std::vector<int64_t>& ids) {
  const adapm_hparams_t& hp = c->hp;
  const double b1 = hp.beta1;
  const int idt = fast ? DT_F32 : DT_F64;
  const OpKind gk = fast ? OP_GEMM_MFMA : OP_GEMM;
  if (ids.empty()) return;
  const std::vector<double> etas = effective_step_sizes(hp.refresh_iters_K);
  const int n_eff = (int)etas.size();
  // Segment length of the Gram-type products of this group.  A workgroup of that launch owns a whole CU (its LDS), so
  // the launch takes (rounds of workgroups over the CUs) x (chunks of the longest workgroup); the scratch of a block
  // holds partial sums for segments of GRAM_SEG_CHUNKS chunks, so only longer segments (fewer of them) are eligible.
  // E.g. 16 layers of the GPT-2-1.5B shape: 25 chunks give 288 workgroups (two rounds on 256 CUs), 34 give 256.
  int gram_seg = GRAM_SEG_CHUNKS;
  if (fast) {
    constexpr int CUS = 256;
    int longest = 1;
    for (int64_t i : ids)
      if (stripe_ok(c->table[i]))
        longest = std::max<int>(longest, (int)((std::max(c->table[i].rows, c->table[i].cols) + 63) / 64));
    int64_t best = -1;
    for (int seg = GRAM_SEG_CHUNKS; seg <= std::max(longest, GRAM_SEG_CHUNKS); ++seg) {
      int64_t wgs = 0;
      int maxlen = 0;
      for (int64_t i : ids) {
        if (!stripe_ok(c->table[i])) continue;
        for (int64_t K : {c->table[i].rows, c->table[i].cols}) {
          const int nch = (int)((K + 63) / 64), nseg = (nch + seg - 1) / seg;
          wgs += nseg;
          maxlen = std::max(maxlen, (nch + nseg - 1) / nseg);
        }
      }
      const int64_t cost = ((wgs + CUS - 1) / CUS) * maxlen;
      if (best < 0 || cost < best) { best = cost; gram_seg = seg; }
    }
  }
  // this group's lists
  const int grp = c->n_groups++;
  c->cp.emplace_back(); c->rub.emplace_back(); c->qt.emplace_back(); c->chol.emplace_back();
  const int chol_id = (int)c->chol.size() - 1;
  c->ru.resize(c->ru.size() + 6);
  const int ru0 = 6 * grp;
  const int img0 = (int)c->img.size(), sit0 = (int)c->sit.size(), gram0 = (int)c->gram.size();
  const int ew_id = fast ? -1 : (int)c->ew.size();
  if (!fast) c->ew.emplace_back();
  auto new_list = [&](bool mfma) {
    c->gemms.emplace_back();
    c->gemms.back().tile = mfma ? 128 : 64;
    return (int)c->gemms.size() - 1;
  };
  std::vector<int> listA(n_eff), listB(n_eff);
  for (int e = 0; e < n_eff; ++e) { listA[e] = new_list(fast); listB[e] = new_list(fast); }
  const int gnorm0 = (int)c->gnorm.size();          // this path's normaliser lists, one per iteration
  if (hp.refresh_normalise) c->gnorm.resize(gnorm0 + n_eff);
  // MFMA path: per GD iteration the images of (R, L^T) and, per rank class, the stripe problems
  constexpr int NXCD = 8;
  struct StripeWork { int prob; int64_t M, K; };
  std::vector<std::vector<StripeWork>> swork(fast ? 6 * n_eff : 0);   // per GD iteration: (rank class, G / G^T)
  if (fast) { c->img.resize(img0 + n_eff); c->sit.resize(sit0 + 6 * n_eff); c->gram.resize(gram0 + n_eff); c->gfin.resize(gram0 + n_eff); }
  auto IMG = [&](int e) -> DevList<ImgItem>& { return c->img[img0 + e]; };
  auto GRAM = [&](int e) -> DevList<GramItem>& { return c->gram[gram0 + e]; };
  // T > 1: the product-preserving orthonormalisation of R follows Alg. 2.  F64 path: inside the group, from the fp64
  // factors in its scratch.  MFMA path: the group stores its factors to the state like a T = 1 step does, and one pass
  // over all blocks re-expresses them in place afterwards (build_plan), whose serial Cholesky kernel would otherwise
  // run once per group on a fraction of the machine.
  const bool group_regauge = hp.refresh_period_T > 1 && !fast;
  const int l_pre = (n_eff == 0 && group_regauge) ? new_list(fast) : -1;
  const int l_epi = fast ? -1 : new_list(false);      // m x n term of eq. 3-4 (the MFMA path never forms it)
  const int l_gram = group_regauge ? new_list(false) : -1;
  const int l_fin = (!fast && (group_regauge || n_eff > 0)) ? new_list(false) : -1;
  for (int64_t i : ids) {
    const adapm_block_t& b = c->table[i];
    const Layout& L = c->lay[i];
    const int m = (int)b.rows, n = (int)b.cols, r = b.rank;
    const int gdt = b.grad_dtype == ADAPM_BF16 ? DT_BF16 : DT_F32;
    const Mat G = mat(SP_GRAD, (int32_t)i, 0, n, 1, gdt);
    const Mat Lp = mat(SP_STATE, 0, L.sL, r, 1, DT_F32), Rp = mat(SP_STATE, 0, L.sR, n, 1, DT_F32);
    auto T = [](const Mat& a) { Mat t = a; t.s0 = a.s1; t.s1 = a.s0; return t; };
    // Where the GD step rides on the stripe products, a workgroup reads and writes only the factor rows behind its own
    // stripe (everything else comes from the images), so the iterations after the first update one working copy in
    // place; the batched GEMM form reads whole rows of the old factor per output tile and alternates two copies.
    const bool inplace = fast && stripe_ok(b);
    auto fL = [&](int which) { return mat(SP_WS, 0, (which && !inplace) ? L.wLb : L.wLa, r, 1, idt); };
    auto fR = [&](int which) { return mat(SP_WS, 0, (which && !inplace) ? L.wRb : L.wRa, n, 1, idt); };
    const Mat P = mat(SP_WS, 0, L.wP, r, 1, idt), S = mat(SP_WS, 0, L.wS, n, 1, idt);
    const Mat Grr = mat(SP_WS, 0, L.wGrr, r, 1, idt), Gpr = mat(SP_WS, 0, L.wGpr, r, 1, idt);
    const Mat Gll = mat(SP_WS, 0, L.wGll, r, 1, idt), Glp = mat(SP_WS, 0, L.wGlp, r, 1, idt);
    Mat Lc = Lp, Rc = Rp;
    GemmProblem p;
    for (int e = 0; e < n_eff; ++e) {
      const double eta = etas[e];
      const Mat Ln = fL(e & 1), Rn = fR(e & 1);
      GemmList& A = c->gemms[listA[e]];
      // thin products of Alg. 2 written without forming L R - m_t:
      //   (L R - m_t) R^T = L (R R^T) - (1-b1) G R^T - b1 L' (R' R^T)
      //   L^T (L R - m_t) = (L^T L) R - (1-b1) L^T G - b1 (L^T L') R'
      if (fast && stripe_ok(b)) {
        // P = G R^T and S = L^T G = (G^T L)^T as stripe products on images of the current factors; the stripes of
        // G^T are 256 columns of G, read with transposing LDS reads
        Mat LcT = T(Lc);
        const int rc = rank_class(r);
        // the images of the first iteration are those of (R_{t-1}, L_{t-1}^T), made by the image kernel and kept for
        // the Gram matrices; the stripes of every iteration write the images of the factors they produce
        auto img_r = [&](int it) { return it == 0 ? L.wIr0 : ((it & 1) ? L.wIr : L.wIr2); };
        auto img_l = [&](int it) { return it == 0 ? L.wIl0 : ((it & 1) ? L.wIl : L.wIl2); };
        const int64_t iR = img_r(e), iL = img_l(e);
        const int64_t iRn = e + 1 < n_eff ? img_r(e + 1) : -1, iLn = e + 1 < n_eff ? img_l(e + 1) : -1;
        if (e == 0) {
          for (int ch = 0; ch < (n + 63) / 64; ++ch) IMG(e).h.push_back(ImgItem{Rc, r, n, ch, rc, iR});
          for (int ch = 0; ch < (m + 63) / 64; ++ch) IMG(e).h.push_back(ImgItem{LcT, r, m, ch, rc, iL});
        }
        // R' R^T with R R^T (contraction over n) and L^T L' with L^T L (over m); longest contraction first
        // ... each with the fragment images of its two results, which the GD step on the stripes multiplies by: image
        // row a, column k = B[k][a] with B = R' R^T, R R^T for L and B = (L^T L')^T, L^T L for R^T
        // a contraction longer than the group's segment length is cut into segments (one workgroup each, partial sums added
        // in segment order by a second small launch): the longest workgroup of a launch then stays short
        auto add_gram = [&](int64_t off_x, int64_t off_s, int64_t o_xs, int64_t o_ss, int64_t i_xs, int64_t i_ss, int K, int tx,
                            int64_t off_part) {
          const int nch = (K + 63) / 64, nseg = (nch + gram_seg - 1) / gram_seg, per = (nch + nseg - 1) / nseg;
          for (int sg = 0; sg < nseg; ++sg)
            GRAM(e).h.push_back(GramItem{off_x, off_s, o_xs, o_ss, i_xs, i_ss, K, r, rc, tx, sg * per, std::min(nch, (sg + 1) * per),
                                         sg, nseg, off_part});
          if (nseg > 1)
            c->gfin[gram0 + e].h.push_back(GramFinItem{off_part, o_xs, o_ss, i_xs, i_ss, r, rc, tx, nseg, off_x == off_s ? 1 : 0, 0});
        };
        add_gram(L.wIr0, iR, L.wGpr, L.wGrr, L.wB[1], L.wB[0], n, 0, L.wGpn);   // R' R^T and R R^T
        add_gram(L.wIl0, iL, L.wGlp, L.wGll, L.wB[3], L.wB[2], m, 1, L.wGpm);   // (L'^T L)^T = L^T L' and L^T L
        // the GD step rides on the stripes: L_new = L + s (-eta L (R R^T) + eta b1 L' (R' R^T) + eta (1-b1) G R^T) on the
        // rows of a stripe of G, R_new likewise on the columns of R behind a stripe of G^T.  The r x r matrices enter
        // as images with row a, column k = B[k][a]: (R R^T)^T and (R' R^T)^T for L; L^T L and L^T L' for R^T.
        const int cls = rc == 32 ? 0 : (rc == 64 ? 1 : 2);
        StripeProb sp;
        memset(&sp, 0, sizeof sp);
        sp.M = m; sp.K = n; sp.r = r; sp.rc = rc;
        sp.upd = 1; sp.off_s = hp.refresh_normalise ? L.wNu : -1;
        sp.c1 = (float)-eta; sp.c2 = (float)(eta * b1); sp.cp = (float)(eta * (1.0 - b1));
        sp.a = G.ref; sp.transpose_out = 0; sp.off_img = iR;
        if (e == 0 && v_fusable(b)) { sp.v_rows = b.v_group_rows; sp.off_v = L.sv; sp.beta2 = hp.beta2; }
        sp.x_cur = Lc.ref; sp.x_prev = Lp.ref; sp.off_b1 = L.wB[0]; sp.off_b2 = L.wB[1]; sp.off_out = Ln.ref.off;
        sp.off_next = iLn; sp.off_timg = -1; sp.off_timg_prev = -1;
        c->sprob.h.push_back(sp);
        swork[6 * e + 2 * cls].push_back(StripeWork{(int)c->sprob.h.size() - 1, m, n});
        sp.M = n; sp.K = m; sp.transpose_out = 1; sp.off_img = iL;
        sp.v_rows = 0;
        sp.x_cur = Rc.ref; sp.x_prev = Rp.ref; sp.off_b1 = L.wB[2]; sp.off_b2 = L.wB[3]; sp.off_out = Rn.ref.off;
        sp.off_next = iRn;
        sp.off_timg = e + 1 == n_eff ? L.wT2 : -1;     // the last iteration leaves the image of R_t^T for the fused update
        sp.off_timg_prev = (e == 0 && hp.bias_correction) ? L.wT1 : -1;   // ... the first one that of R_{t-1}^T
        c->sprob.h.push_back(sp);
        swork[6 * e + 2 * cls + 1].push_back(StripeWork{(int)c->sprob.h.size() - 1, n, m});
      } else {
        p = problem(m, r); p.A1 = G; p.B1 = T(Rc); p.K1 = n; p.a1 = 1; p.scale_g = 1; p.Out = P; add_problem(A, p);
        p = problem(r, n); p.A1 = T(Lc); p.B1 = G; p.K1 = m; p.a1 = 1; p.scale_g = 1; p.Out = S; add_problem(A, p);
      }
      if (!(fast && stripe_ok(b))) {
        p = problem(r, r); p.A1 = Rc; p.B1 = T(Rc); p.K1 = n; p.a1 = 1; p.Out = Grr; add_problem(A, p);
        p = problem(r, r); p.A1 = Rp; p.B1 = T(Rc); p.K1 = n; p.a1 = 1; p.Out = Gpr; add_problem(A, p);
        p = problem(r, r); p.A1 = T(Lc); p.B1 = Lc; p.K1 = m; p.a1 = 1; p.Out = Gll; add_problem(A, p);
        p = problem(r, r); p.A1 = T(Lc); p.B1 = Lp; p.K1 = m; p.a1 = 1; p.Out = Glp; add_problem(A, p);
      }
      GemmList& Bl = c->gemms[listB[e]];
      // optional: both updates of this iteration take eta / max(||R R^T||_F, ||L^T L||_F), a device scalar
      const int64_t off_s = hp.refresh_normalise ? L.wNu : -1;
      if (hp.refresh_normalise) c->gnorm[gnorm0 + e].h.push_back(GnormItem{L.wGrr, L.wGll, L.wNu, r, idt});
      if (!(fast && stripe_ok(b))) {
        p = problem(m, r);
        p.A1 = Lc; p.B1 = Grr; p.K1 = r; p.a1 = -eta;
        p.A2 = Lp; p.B2 = Gpr; p.K2 = r; p.a2 = eta * b1;
        p.X = Lc; p.g = 1.0; p.Y = P; p.d = eta * (1.0 - b1); p.Out = Ln; p.off_s = off_s;
        add_problem(Bl, p);
        p = problem(r, n);
        p.A1 = Gll; p.B1 = Rc; p.K1 = r; p.a1 = -eta;
        p.A2 = Glp; p.B2 = Rp; p.K2 = r; p.a2 = eta * b1;
        p.X = Rc; p.g = 1.0; p.Y = S; p.d = eta * (1.0 - b1); p.Out = Rn; p.off_s = off_s;
        add_problem(Bl, p);
      }
      Lc = Ln; Rc = Rn;
    }
    if (l_pre >= 0) {      // no effective iteration but an in-place re-gauge ahead: work on a copy
      p = problem(m, r); p.X = Lp; p.g = 1.0; p.Out = fL(0); add_problem(c->gemms[l_pre], p);
      p = problem(r, n); p.X = Rp; p.g = 1.0; p.Out = fR(0); add_problem(c->gemms[l_pre], p);
      Lc = fL(0); Rc = fR(0);
    }
    if (fast) {
      // eq. 3-4 fused into the update: L'R' - L R (or L R without the correction) is built tile by tile
      RuBlockDev d;
      memset(&d, 0, sizeof d);
      d.block = (int32_t)i; d.m = m; d.n = n; d.r = r; d.rc = rank_class(r);
      if (b.v_mode == ADAPM_V_ELEMENT) { d.v_kind = 0; d.v_group_rows = 1; }
      else { d.v_kind = 2; d.v_group_rows = b.v_mode == ADAPM_V_WHOLE ? (int32_t)b.rows : b.v_group_rows; }
      d.param_dtype = b.param_dtype; d.lr_scale = b.lr_scale; d.wd = b.weight_decay;
      d.a1 = hp.bias_correction ? 1.f : 0.f; d.a2 = hp.bias_correction ? -1.f : 1.f;
      d.l1 = Lp.ref; d.l2 = Lc.ref; d.q1 = Rp.ref; d.q2 = Rc.ref; d.off_img1 = L.wT1; d.off_img2 = L.wT2; d.off_v = L.sv;
      c->rub[grp].h.push_back(d);
      for (int ch = 0; ch < (n + 63) / 64; ++ch) {
        if (hp.bias_correction && !(stripe_ok(b) && n_eff > 0)) c->qt[grp].h.push_back(ImgItem{Rp, r, n, ch, d.rc, L.wT1});
        if (!(stripe_ok(b) && n_eff > 0)) c->qt[grp].h.push_back(ImgItem{Rc, r, n, ch, d.rc, L.wT2});   // else: written by the stripes
      }
    } else {
      // m x n low-rank term of m^c (eq. 4): C = L'R' - L R, or L R without the correction
      const Mat C = mat(SP_WS, 0, L.wC, n, 1, DT_F32);
      p = problem(m, n);
      if (hp.bias_correction) {
        p.A1 = Lp; p.B1 = Rp; p.K1 = r; p.a1 = 1.0;
        p.A2 = Lc; p.B2 = Rc; p.K2 = r; p.a2 = -1.0;
      } else {
        p.A1 = Lc; p.B1 = Rc; p.K1 = r; p.a1 = 1.0;
      }
      p.Out = C;
      add_problem(c->gemms[l_epi], p);
      for (int64_t s0 = 0; s0 < (int64_t)m * n; s0 += EW_CHUNK)
        c->ew[ew_id].h.push_back(EwItem{s0, (int32_t)i, (int32_t)std::min<int64_t>(EW_CHUNK, (int64_t)m * n - s0)});
    }
    if (fast && hp.refresh_period_T > 1) {
      // the pass over all blocks that follows the last group: Gram matrix of the stored R in fp64, Cholesky, in place
      const Mat G64 = mat(SP_WS, 0, L.wG64, r, 1, DT_F64);
      p = problem(r, r); p.A1 = Rp; p.B1 = T(Rp); p.K1 = n; p.a1 = 1.0; p.Out = G64;
      add_problem(c->gemms[c->rg_gram], p, 0, true);
      c->chol[c->rg_chol].h.push_back(CholItem{L.wG64, L.wCinv, r, 0});
      for (int f = 0; f < n; f += 64) c->rg_apply.h.push_back(RegaugeItem{L.sR, L.wCinv, r, n, f, 0});
      for (int f = 0; f < m; f += 64) c->rg_apply.h.push_back(RegaugeItem{L.sL, L.wG64, r, m, f, 1});
    }
    if (group_regauge) {
      // product-preserving orthonormalisation of R, always in fp64
      const Mat G64 = mat(SP_WS, 0, L.wG64, r, 1, DT_F64), Cinv = mat(SP_WS, 0, L.wCinv, r, 1, DT_F64);
      p = problem(r, r); p.A1 = Rc; p.B1 = T(Rc); p.K1 = n; p.a1 = 1.0; p.Out = G64;
      add_problem(c->gemms[l_gram], p, 0, true);      // the Cholesky factorisation reads the lower triangle only
      c->chol[chol_id].h.push_back(CholItem{L.wG64, L.wCinv, r, 0});
      // C^-1 and C are lower triangular
      p = problem(r, n); p.A1 = Cinv; p.B1 = Rc; p.K1 = r; p.a1 = 1.0; p.tri = 1; p.Out = Rp; add_problem(c->gemms[l_fin], p);
      p = problem(m, r); p.A1 = Lc; p.B1 = G64; p.K1 = r; p.a1 = 1.0; p.tri = 2; p.Out = Lp; add_problem(c->gemms[l_fin], p);
    } else if (n_eff > 0) {
      if (fast) {
        for (int64_t f = 0; f < (int64_t)m * r; f += COPY_CHUNK)
          c->cp[grp].h.push_back(CopyItem{Lc.ref, Lp.ref, f, (int32_t)std::min<int64_t>(COPY_CHUNK, (int64_t)m * r - f), 0});
        for (int64_t f = 0; f < (int64_t)r * n; f += COPY_CHUNK)
          c->cp[grp].h.push_back(CopyItem{Rc.ref, Rp.ref, f, (int32_t)std::min<int64_t>(COPY_CHUNK, (int64_t)r * n - f), 0});
      } else {
        p = problem(m, r); p.X = Lc; p.g = 1.0; p.Out = Lp; add_problem(c->gemms[l_fin], p);
        p = problem(r, n); p.X = Rc; p.g = 1.0; p.Out = Rp; add_problem(c->gemms[l_fin], p);
      }
    }
  }
  // stripes of one problem go to one XCD (workgroup i runs on XCD i mod 8) so that they share the image
  // through its L2; longest contraction first, problems dealt to the least loaded XCD
  for (size_t w = 0; w < swork.size(); ++w) {
    std::vector<StripeWork>& v = swork[w];
    std::stable_sort(v.begin(), v.end(), [](const StripeWork& a, const StripeWork& b) {
      if (a.K != b.K) return a.K > b.K;
      return a.M > b.M;
    });
    std::vector<StripeItem> per[NXCD];
    double load[NXCD] = {0};
    for (const StripeWork& sw : v) {
      int x = 0;
      for (int k = 1; k < NXCD; ++k) if (load[k] < load[x]) x = k;
      for (int64_t r0 = 0; r0 < sw.M; r0 += 256) per[x].push_back(StripeItem{sw.prob, (int32_t)r0});   // two stripes per workgroup
      load[x] += (double)sw.M * sw.K;
    }
    size_t longest = 0;
    for (auto& q : per) longest = std::max(longest, q.size());
    for (size_t q = 0; q < longest; ++q)
      for (int x = 0; x < NXCD; ++x) c->sit[sit0 + w].h.push_back(q < per[x].size() ? per[x][q] : StripeItem{-1, 0});
  }
  std::vector<Op>& seq = c->seq_refresh;
  for (int e = 0; e < n_eff; ++e) {
    const bool stripes = fast && !GRAM(e).h.empty();
    if (stripes) {
      if (!IMG(e).h.empty()) seq.push_back(Op{OP_QFIMG, img0 + e, 0, 0, "alg2_factor_images"});
      std::stable_sort(GRAM(e).h.begin(), GRAM(e).h.end(),
                       [](const GramItem& a, const GramItem& b) { return a.c1 - a.c0 > b.c1 - b.c0; });
      seq.push_back(Op{OP_GRAM, gram0 + e, 0, 0, "alg2_gram_products"});
      if (!c->gfin[gram0 + e].h.empty()) seq.push_back(Op{OP_GRAM_FIN, gram0 + e, 0, 0, "alg2_gram_segments_sum"});
    }
    if (!c->gemms[listA[e]].tiles.empty())
      seq.push_back(Op{gk, listA[e], 0, 0, fast ? "alg2_products_mfma" : "alg2_products_f64"});
    if (hp.refresh_normalise) seq.push_back(Op{OP_GNORM, gnorm0 + e, 0, 0, "alg2_step_normaliser"});
    if (stripes) {
      // both streaming products of the iteration and, behind each stripe, the GD step on the factor rows it covers
      static const char* names[6] = {"alg2_stripe_step_L_r32", "alg2_stripe_step_R_r32", "alg2_stripe_step_L_r64",
                                     "alg2_stripe_step_R_r64", "alg2_stripe_step_L_r128", "alg2_stripe_step_R_r128"};
      for (int k = 0; k < 6; ++k)
        if (!c->sit[sit0 + 6 * e + k].h.empty()) seq.push_back(Op{OP_STRIPE, sit0 + 6 * e + k, 0, 0, names[k]});
    }
    if (!c->gemms[listB[e]].tiles.empty())
      seq.push_back(Op{gk, listB[e], 0, 0, fast ? "alg2_update_mfma" : "alg2_update_f64"});
  }
  if (l_pre >= 0) seq.push_back(Op{gk, l_pre, 0, 0, "copy_factors"});
  const float cG = hp.bias_correction ? 1.f : 0.f;
  const float cC = hp.bias_correction ? (float)(b1 / (1.0 - b1)) : 1.f;
  if (fast) {
    // stripes of the fused update, per (rank class, parameter type), whole blocks dealt to XCDs
    if (!c->qt[grp].h.empty()) seq.push_back(Op{OP_QTIMG, grp, 0, 0, "update_factor_images"});
    for (int cls = 0; cls < 6; ++cls) {
      const int rank = 32 << (cls >> 1);
      const int pdt = (cls & 1) ? ADAPM_BF16 : ADAPM_F32;
      std::vector<size_t> ids;
      const std::vector<RuBlockDev>& rubs = c->rub[grp].h;
      for (size_t k = 0; k < rubs.size(); ++k)
        if (rubs[k].rc == rank && rubs[k].param_dtype == pdt) ids.push_back(k);
      if (ids.empty()) continue;
      std::stable_sort(ids.begin(), ids.end(), [&](size_t a, size_t b2) {
        const RuBlockDev &x = rubs[a], &y = rubs[b2];
        if (x.n != y.n) return x.n > y.n;
        return (double)x.m * x.n > (double)y.m * y.n;
      });
      std::vector<ProjItem> per[NXCD];
      double load[NXCD] = {0};
      for (size_t k : ids) {
        int x = 0;
        for (int q = 1; q < NXCD; ++q) if (load[q] < load[x]) x = q;
        const RuBlockDev& d = rubs[k];
        for (int r0 = 0; r0 < d.m; r0 += 128) per[x].push_back(ProjItem{(int32_t)k, r0});
        load[x] += (double)d.m * d.n;
      }
      size_t longest = 0;
      for (auto& q : per) longest = std::max(longest, q.size());
      for (size_t q = 0; q < longest; ++q)
        for (int x = 0; x < NXCD; ++x) c->ru[ru0 + cls].h.push_back(q < per[x].size() ? per[x][q] : ProjItem{-1, 0});
      static const char* names[3] = {"fused_refresh_update_r32", "fused_refresh_update_r64", "fused_refresh_update_r128"};
      seq.push_back(Op{OP_REFRESH_UPDATE, ru0 + cls, cG, cC, names[cls >> 1], grp});
    }
  } else {
    seq.push_back(Op{gk, l_epi, 0, 0, "reconstruct_f64"});
    seq.push_back(Op{OP_UPDATE, ew_id, cG, cC, "update_lowrank"});
  }
  if (l_gram >= 0) {
    seq.push_back(Op{OP_GEMM, l_gram, 0, 0, "regauge_gram_f64"});
    seq.push_back(Op{OP_CHOL, chol_id, 0, 0, "regauge_cholesky_f64"});
  }
  if (l_fin >= 0 && !c->gemms[l_fin].tiles.empty()) {
    const bool f64_fin = group_regauge;
    seq.push_back(Op{f64_fin ? OP_GEMM : gk, l_fin, 0, 0, f64_fin ? "regauge_apply_f64" : "store_factors"});
  }
  if (fast && !c->cp[grp].h.empty()) seq.push_back(Op{OP_COPY, grp, 0, 0, "store_factors"});
}

// step with R held, F64 path: four batched GEMM launches and the update kernel
// `ids`: one group of blocks (the scratch of a group is reused by the next); ew_id: the group's element-wise list
void plan_lowrank_project_f64(adapm_ctx* c, const std::vector<int64_t>& ids, int ew_id) {
  const adapm_hparams_t& hp = c->hp;
  const double b1 = hp.beta1;
  if (ids.empty()) return;
  auto new_list = [&]() { c->gemms.emplace_back(); return (int)c->gemms.size() - 1; };
  const int l_p = new_list(), l_d = new_list(), l_l = new_list(), l_c = new_list();
  for (int64_t i : ids) {
    const adapm_block_t& b = c->table[i];
    const Layout& L = c->lay[i];
    const int m = (int)b.rows, n = (int)b.cols, r = b.rank;
    const int gdt = b.grad_dtype == ADAPM_BF16 ? DT_BF16 : DT_F32;
    const Mat G = mat(SP_GRAD, (int32_t)i, 0, n, 1, gdt);
    const Mat Ls = mat(SP_STATE, 0, L.sL, r, 1, DT_F32), Q = mat(SP_STATE, 0, L.sR, n, 1, DT_F32);
    Mat Qt = Q; Qt.s0 = Q.s1; Qt.s1 = Q.s0;
    const Mat P = mat(SP_WS, 0, L.wP, r, 1, DT_F64), D = mat(SP_WS, 0, L.wLa, r, 1, DT_F64);
    const Mat C = mat(SP_WS, 0, L.wC, n, 1, DT_F32);
    GemmProblem p;
    p = problem(m, r); p.A1 = G; p.B1 = Qt; p.K1 = n; p.a1 = 1.0; p.scale_g = 1; p.Out = P; add_problem(c->gemms[l_p], p);
    // L_t = b1 L' + (1-b1) G Q^T;  m^c = G + b1 (L' - G Q^T) Q   (or L_t Q without the correction)
    p = problem(m, r); p.X = Ls; p.Y = P; p.Out = D;
    if (hp.bias_correction) { p.g = b1; p.d = -b1; } else { p.g = b1; p.d = 1.0 - b1; }
    add_problem(c->gemms[l_d], p);
    p = problem(m, r); p.X = Ls; p.g = b1; p.Y = P; p.d = 1.0 - b1; p.Out = Ls; add_problem(c->gemms[l_l], p);
    p = problem(m, n); p.A1 = D; p.B1 = Q; p.K1 = r; p.a1 = 1.0; p.Out = C; add_problem(c->gemms[l_c], p);
  }
  std::vector<Op>& seq = c->seq_project;
  seq.push_back(Op{OP_GEMM, l_p, 0, 0, "project_f64"});
  seq.push_back(Op{OP_GEMM, l_d, 0, 0, "project_residual_f64"});
  seq.push_back(Op{OP_GEMM, l_l, 0, 0, "project_store_L_f64"});
  seq.push_back(Op{OP_GEMM, l_c, 0, 0, "reconstruct_f64"});
  seq.push_back(Op{OP_UPDATE, ew_id, hp.bias_correction ? 1.f : 0.f, 1.f, "update_lowrank"});
}

// step with R held, MFMA path: Q^T split once, then one fused launch per rank class.  Stripes of one
// block are placed on one XCD (workgroup i runs on XCD i mod 8) so that they share Q through its L2.
void plan_lowrank_project_fast(adapm_ctx* c) {
  const int64_t nb = (int64_t)c->table.size();
  constexpr int NXCD = 8;
  std::vector<int64_t> lr_of(nb, -1);
  for (int64_t i = 0; i < nb; ++i) {
    const adapm_block_t& b = c->table[i];
    const Layout& L = c->lay[i];
    if (L.path != PATH_FAST) continue;
    LrBlockDev d;
    memset(&d, 0, sizeof d);
    d.block = (int32_t)i; d.m = (int32_t)b.rows; d.n = (int32_t)b.cols; d.r = b.rank; d.rc = rank_class(b.rank);
    d.off_L = L.sL; d.off_Q = L.sR; d.off_v = L.sv; d.off_Qf = L.wQf; d.off_Timg = L.wTimg;
    if (b.v_mode == ADAPM_V_ELEMENT) { d.v_kind = 0; d.v_group_rows = 1; }
    else if (v_fusable(b)) { d.v_kind = 1; d.v_group_rows = b.v_group_rows; }
    else { d.v_kind = 2; d.v_group_rows = b.v_mode == ADAPM_V_WHOLE ? (int32_t)b.rows : b.v_group_rows; }
    d.param_dtype = b.param_dtype; d.lr_scale = b.lr_scale; d.wd = b.weight_decay;
    lr_of[i] = (int64_t)c->lrb.h.size();
    c->lrb.h.push_back(d);
    for (int ch = 0; ch < (int)((b.cols + 63) / 64); ++ch) c->qs.h.push_back(QsItem{(int32_t)lr_of[i], ch});
  }
  if (c->lrb.h.empty()) return;
  std::vector<Op>& seq = c->seq_project;
  // the bf16 (hi, lo) copies of Q are rebuilt after every run of Alg. 2 (and whenever the caller
  // hands in a different workspace); steps with R held reuse them
  c->seq_refresh.push_back(Op{OP_QSPLIT, 0, 0, 0, "split_Q"});
  seq.push_back(Op{OP_QSPLIT, 1, 0, 0, "split_Q"});
  for (int cls = 0; cls < 12; ++cls) {      // (rank 32 / 64 / 128) x (fp32 / bf16 parameters) x (blockwise / per-element v)
    const int rank = 32 << ((cls >> 1) % 3);
    const int pdt = (cls & 1) ? ADAPM_BF16 : ADAPM_F32;
    const bool vel = cls >= 6;
    // blocks of rank class 128 with bf16 parameters, a blockwise v and short rows go to the kernel that reads G once
    auto keeps = [&](const adapm_block_t& b) {
      if (rank != 128 || pdt != ADAPM_BF16 || vel || !c->keep_enabled) return false;
      if (b.cols % 8 != 0 || b.cols > proj_keep_max_cols()) return false;
      return !v_fusable(b) || proj_keep_rows() % b.v_group_rows == 0;      // groups finished inside the stripe must fit it
    };
    for (int pass = 0; pass < 2; ++pass) {       // 0: the two-read kernel (long rows first), 1: the kernel that keeps G on chip
      const int rows_per = pass ? proj_keep_rows() : 128;
      std::vector<int64_t> ids;
      for (int64_t i = 0; i < nb; ++i)
        if (lr_of[i] >= 0 && rank_class(c->table[i].rank) == rank && c->table[i].param_dtype == pdt &&
            (c->table[i].v_mode == ADAPM_V_ELEMENT) == vel && keeps(c->table[i]) == (pass == 1))
          ids.push_back(i);
      if (ids.empty()) continue;
      // longest rows first; whole blocks dealt to the least loaded XCD
      std::stable_sort(ids.begin(), ids.end(), [&](int64_t a, int64_t b) {
        const double ca = (double)c->table[a].rows * c->table[a].cols, cb = (double)c->table[b].rows * c->table[b].cols;
        if (c->table[a].cols != c->table[b].cols) return c->table[a].cols > c->table[b].cols;
        return ca > cb;
      });
      std::vector<ProjItem> per[NXCD];
      double load[NXCD] = {0};
      for (int64_t i : ids) {
        int x = 0;
        for (int k = 1; k < NXCD; ++k) if (load[k] < load[x]) x = k;
        const adapm_block_t& b = c->table[i];
        for (int64_t r0 = 0; r0 < b.rows; r0 += rows_per) per[x].push_back(ProjItem{(int32_t)lr_of[i], (int32_t)r0});
        load[x] += (double)b.rows * b.cols;
      }
      size_t longest = 0;
      for (auto& v : per) longest = std::max(longest, v.size());
      std::vector<ProjItem>& out = pass ? c->proj_keep.h : c->proj[cls].h;
      for (size_t q = 0; q < longest; ++q)
        for (int x = 0; x < NXCD; ++x) out.push_back(q < per[x].size() ? per[x][q] : ProjItem{-1, 0});
      static const char* names[3] = {"fused_project_r32", "fused_project_r64", "fused_project_r128"};
      if (pass) seq.push_back(Op{OP_PROJ_KEEP, 0, 0, 0, "fused_project_keep_r128"});
      else seq.push_back(Op{OP_PROJ, cls, 0, 0, names[(cls >> 1) % 3]});
    }
  }
}

// Lay out state / workspace and build every work list.
// Scratch of one low-rank block while its group runs Alg. 2 (and, on the F64 path, a step with R held): laid out
// from `base` on; returns the end.  dry = true only measures.
size_t layout_block_scratch(const adapm_block_t& b, const adapm_hparams_t& hp, Layout& L, size_t base, bool dry) {
  size_t wo = base;
  Layout tmp;
  Layout& T = dry ? tmp : L;
  auto walloc = [&](size_t bytes) { int64_t o = (int64_t)wo; wo += align_up(bytes); return o; };
  const int64_t m = b.rows, n = b.cols, r = b.rank;
  const bool fast = L.path == PATH_FAST, stripes = fast && stripe_ok(b);
  // F64 path: every intermediate of a step stays in fp64, only the state is rounded to fp32
  const size_t es = fast ? 4 : 8;
  T.wLa = walloc(es * m * r); T.wRa = walloc(es * r * n);
  // the second working copy of the factors: only where the GD step runs as batched GEMMs (see plan_lowrank_refresh)
  if (!stripes) { T.wLb = walloc(es * m * r); T.wRb = walloc(es * r * n); }
  // G R^T and L^T G: blocks whose GD step rides on the stripe products never store them
  if (!stripes) { T.wP = walloc(es * m * r); T.wS = walloc(es * r * n); }
  T.wGrr = walloc(es * r * r); T.wGpr = walloc(es * r * r);
  T.wGll = walloc(es * r * r); T.wGlp = walloc(es * r * r);
  if (hp.refresh_period_T > 1 && !fast) { T.wG64 = walloc(8 * r * r); T.wCinv = walloc(8 * r * r); }
  T.wNu = walloc(8);
  if (fast) {
    T.wT1 = walloc(proj_timg_bytes(rank_class((int)r), (int)n));
    T.wT2 = walloc(proj_timg_bytes(rank_class((int)r), (int)n));
  } else {
    T.wC = walloc(4 * m * n);
  }
  if (stripes) {
    T.wIr = walloc(proj_qf_bytes(rank_class((int)r), (int)n));
    T.wIl = walloc(proj_qf_bytes(rank_class((int)r), (int)m));
    T.wIr2 = walloc(proj_qf_bytes(rank_class((int)r), (int)n));
    T.wIl2 = walloc(proj_qf_bytes(rank_class((int)r), (int)m));
    T.wIr0 = walloc(proj_qf_bytes(rank_class((int)r), (int)n));
    T.wIl0 = walloc(proj_qf_bytes(rank_class((int)r), (int)m));
    for (int k = 0; k < 4; ++k) T.wB[k] = walloc(proj_qf_bytes(rank_class((int)r), (int)r));
    const size_t rc = (size_t)rank_class((int)r);
    if (gram_segments(n) > 1) T.wGpn = walloc((size_t)gram_segments(n) * 2 * rc * rc * 4);
    if (gram_segments(m) > 1) T.wGpm = walloc((size_t)gram_segments(m) * 2 * rc * rc * 4);
  }
  return wo;
}

// Lay out state / workspace and build every work list.
//
// Workspace = [what has to survive from step to step or is global | scratch of ONE group of low-rank blocks].
// Alg. 2 (and the F64 form of the step with R held) runs group by group, every group from its first launch to its
// last before the next one starts in the same scratch, so that the scratch scales with a group, not with the
// model.  A group holds as many blocks (in table order, per contraction path) as fit a budget chosen so that the
// whole workspace stays below the size of the optimizer state; the largest single block sets the minimum.
void build_plan(adapm_ctx* c) {
  const int64_t nb = (int64_t)c->table.size();
  const adapm_hparams_t& hp = c->hp;
  c->lay.assign(nb, Layout());
  size_t so = 0, wo = 0;

  for (int64_t i = 0; i < nb; ++i) {
    const adapm_block_t& b = c->table[i];
    Layout& L = c->lay[i];
    const int64_t m = b.rows, n = b.cols, r = b.rank;
    auto salloc = [&](size_t bytes) { int64_t o = (int64_t)so; so += align_up(bytes); return o; };
    auto walloc = [&](size_t bytes) { int64_t o = (int64_t)wo; wo += align_up(bytes); return o; };
    L.path = path_of(b, hp);
    if (b.mom_mode == ADAPM_MOM_LOWRANK) {
      L.sL = salloc(4 * m * r);
      L.sR = salloc(4 * r * n);
      if (L.path == PATH_FAST && hp.refresh_period_T > 1) {
        L.wG64 = walloc(8 * r * r);        // Gram matrix of R, then its Cholesky factor C, and C^-1: the pass over all
        L.wCinv = walloc(8 * r * r);       // blocks that follows the last group's Alg. 2
      }
      c->n_lowrank++;
    } else if (b.mom_mode == ADAPM_MOM_FULL) {
      L.sm = salloc(4 * m * n);
    }
    L.nv = num_v(b);
    L.sv = salloc(4 * L.nv);
  }
  c->state_bytes = so;
  c->ew.clear();
  c->ew.emplace_back();          // list 0: full / no momentum blocks

  // device block table, element-wise chunks, v statistics
  int64_t npart = 0;
  for (int64_t i = 0; i < nb; ++i) {
    const adapm_block_t& b = c->table[i];
    const Layout& L = c->lay[i];
    BlockDev d;
    d.numel = b.rows * b.cols;
    d.group_elems = group_elems(b);
    d.off_m = L.sm; d.off_v = L.sv; d.off_C = -1;      // off_C: set when the block's group is laid out
    d.param_dtype = b.param_dtype; d.grad_dtype = b.grad_dtype;
    d.mom_mode = b.mom_mode; d.v_mode = b.v_mode;
    d.lr_scale = b.lr_scale; d.wd = b.weight_decay;
    c->blocks.h.push_back(d);
    // full / no momentum blocks with a blockwise v whose groups fit a wavefront's registers: one fused kernel
    const bool grouped = L.path == PATH_NONE && b.v_mode != ADAPM_V_ELEMENT && d.group_elems <= GRP_MAX_ELEMS &&
                         d.group_elems % 8 == 0 && b.grad_dtype == ADAPM_BF16 && b.param_dtype == ADAPM_BF16;
    if (grouped) {
      const int64_t per = std::max<int64_t>(4, 32768 / d.group_elems);      // groups per workgroup (4 waves)
      for (int64_t g0 = 0; g0 < L.nv; g0 += per)
        c->grp.h.push_back(GrpItem{g0, (int32_t)i, (int32_t)std::min<int64_t>(per, L.nv - g0)});
      continue;
    }
    // low-rank blocks are updated by their group's launches (element-wise on the F64 path, fused stripe kernels on
    // the MFMA path)
    if (L.path == PATH_NONE) {
      for (int64_t s = 0; s < d.numel; s += EW_CHUNK)
        c->ew[0].h.push_back(EwItem{s, (int32_t)i, (int32_t)std::min<int64_t>(EW_CHUNK, d.numel - s)});
    }
    if (b.v_mode != ADAPM_V_ELEMENT) {
      // on the MFMA path with T > 1 the fused kernel finishes fusable groups itself on steps with R held (list 1: only
      // steps that run Alg. 2), and where Alg. 2 streams G in stripes its first GD iteration does so (no list at all)
      const int which = (L.path == PATH_FAST && hp.refresh_period_T > 1 && v_fusable(b)) ? 1 : 0;
      const bool in_stripes = L.path == PATH_FAST && v_fusable(b) && stripe_ok(b) &&
                              !effective_step_sizes(hp.refresh_iters_K).empty() && (which == 1 || hp.refresh_period_T == 1);
      const int64_t ge = d.group_elems;
      for (int64_t g = 0; g < (in_stripes ? 0 : L.nv); ++g) {
        if (ge <= VS_CHUNK) {
          c->vs[which].h.push_back(VsItem{g * ge, g, (int32_t)i, (int32_t)ge, 1, 0});
        } else {
          const int64_t np = (ge + VS_CHUNK - 1) / VS_CHUNK;
          c->vf[which].h.push_back(VfItem{npart, g, (int32_t)i, (int32_t)np});
          for (int64_t p = 0; p < np; ++p)
            c->vs[which].h.push_back(VsItem{g * ge + p * VS_CHUNK, npart + p, (int32_t)i,
                                            (int32_t)std::min<int64_t>(VS_CHUNK, ge - p * VS_CHUNK), 0, 0});
          npart += np;
        }
      }
    }
    if (b.mom_mode == ADAPM_MOM_LOWRANK && hp.seed != 0) {
      SketchItem s;
      s.off_R = L.sR; s.count = (int64_t)b.rank * b.cols;
      s.key = mix64(hp.seed ^ mix64((uint64_t)i));
      s.amp = (float)(std::sqrt(3.0) / (std::sqrt((double)b.cols) + std::sqrt((double)b.rank)) * std::ldexp(1.0, -23));
      s.pad = 0;
      c->sk.h.push_back(s);
    }
  }
  if (npart > 0) { c->off_partials = (int64_t)wo; wo += align_up(8 * (size_t)npart); }
  // global gradient norm: one partial sum per piece of every gradient, then norm and factor (two floats)
  for (int64_t i = 0; i < nb; ++i) {
    const int64_t numel = c->table[i].rows * c->table[i].cols;
    for (int64_t s0 = 0; s0 < numel; s0 += VS_CHUNK)
      c->gn.h.push_back(VsItem{s0, (int64_t)c->gn.h.size(), (int32_t)i, (int32_t)std::min<int64_t>(VS_CHUNK, numel - s0), 0, 0});
  }
  c->off_gn_partials = (int64_t)wo; wo += align_up(8 * c->gn.h.size());
  c->off_gn_out = (int64_t)wo; wo += align_up(8);
  // kept between two runs of Alg. 2: the bf16 (hi, lo) images of the held R, last in this part of the workspace.
  // A step that runs Alg. 2 rebuilds them at its end and reads them nowhere, so where no other step needs scratch
  // (the F64 form of the step with R held does) the groups' scratch starts where the images start.
  const size_t images_at = wo;
  bool scratch_in_held_steps = false;
  for (int64_t i = 0; i < nb; ++i) {
    const adapm_block_t& b = c->table[i];
    Layout& L = c->lay[i];
    if (L.path == PATH_F64) scratch_in_held_steps = true;
    if (L.path != PATH_FAST || hp.refresh_period_T <= 1) continue;
    auto walloc = [&](size_t bytes) { int64_t o = (int64_t)wo; wo += align_up(bytes); return o; };
    L.wQf = walloc(proj_qf_bytes(rank_class(b.rank), (int)b.cols));
    L.wTimg = walloc(proj_timg_bytes(rank_class(b.rank), (int)b.cols));
  }
  const size_t images_end = wo;
  const size_t persistent = scratch_in_held_steps ? images_end : images_at;     // where the groups' scratch starts

  // ---- every step starts with the v statistics and the full / no-momentum blocks
  for (int kind = 0; kind < 2; ++kind) {
    std::vector<Op>& seq = kind == 0 ? c->seq_refresh : c->seq_project;
    if (!c->vs[0].h.empty()) seq.push_back(Op{OP_VSTAT, 0, 0, 0, "v_statistics"});
    if (!c->vf[0].h.empty()) seq.push_back(Op{OP_VFINAL, 0, 0, 0, "v_statistics_fold"});
    if (kind == 0) {
      if (!c->vs[1].h.empty()) seq.push_back(Op{OP_VSTAT, 1, 0, 0, "v_statistics"});
      if (!c->vf[1].h.empty()) seq.push_back(Op{OP_VFINAL, 1, 0, 0, "v_statistics_fold"});
    }
    if (!c->ew[0].h.empty()) seq.push_back(Op{OP_UPDATE, 0, 0, 0, "update_full"});
    if (!c->grp.h.empty()) seq.push_back(Op{OP_UPDATE_GROUPED, 0, 0, 0, "update_full_grouped"});
  }
  c->ws_bytes = images_end;
  if (c->n_lowrank == 0) return;

  // ---- groups of low-rank blocks: scratch budget, then per group the layout and the launches
  size_t largest = 0;
  for (int64_t i = 0; i < nb; ++i)
    if (c->lay[i].path != PATH_NONE) largest = std::max(largest, layout_block_scratch(c->table[i], hp, c->lay[i], 0, true));
  const size_t floor_bytes = (size_t)32 << 20;
  size_t budget = c->state_bytes > persistent + floor_bytes ? c->state_bytes - persistent : floor_bytes;
  budget = std::max(budget - budget / 16, largest);          // a margin below the state size; at least one block
  size_t scratch_max = 0;
  if (hp.refresh_period_T > 1) {
    c->gemms.emplace_back();
    c->rg_gram = (int)c->gemms.size() - 1;
    c->chol.emplace_back();              // groups append theirs behind it (plan_lowrank_refresh indexes by its own position)
    c->rg_chol = (int)c->chol.size() - 1;
  }
  for (int path : {PATH_F64, PATH_FAST}) {
    // groups of about equal size: as few as the budget allows, none above it
    size_t total = 0;
    for (int64_t i = 0; i < nb; ++i)
      if (c->lay[i].path == path) total += layout_block_scratch(c->table[i], hp, c->lay[i], 0, true);
    const size_t n_groups = (total + budget - 1) / budget;
    const size_t target = n_groups ? (total + n_groups - 1) / n_groups : 0;
    std::vector<int64_t> ids;
    size_t used = 0;
    auto flush = [&]() {
      if (ids.empty()) return;
      size_t at = persistent;
      for (int64_t i : ids) {
        at = layout_block_scratch(c->table[i], hp, c->lay[i], at, false);
        c->blocks.h[i].off_C = c->lay[i].wC;
      }
      scratch_max = std::max(scratch_max, at - persistent);
      const int ew_before = (int)c->ew.size();
      plan_lowrank_refresh(c, path == PATH_FAST, ids);
      if (hp.refresh_period_T > 1 && path == PATH_F64) plan_lowrank_project_f64(c, ids, ew_before);
      ids.clear();
      used = 0;
    };
    for (int64_t i = 0; i < nb; ++i) {
      if (c->lay[i].path != path) continue;
      const size_t need = layout_block_scratch(c->table[i], hp, c->lay[i], 0, true);
      if (!ids.empty() && (used + need > budget || used >= target)) flush();
      ids.push_back(i);
      used += need;
    }
    flush();
  }
  c->ws_bytes = std::max(images_end, persistent + scratch_max);
  if (hp.refresh_period_T > 1 && !c->rg_apply.h.empty()) {
    c->seq_refresh.push_back(Op{OP_GEMM, c->rg_gram, 0, 0, "regauge_gram_f64"});
    c->seq_refresh.push_back(Op{OP_CHOL, c->rg_chol, 0, 0, "regauge_cholesky_f64"});
    c->seq_refresh.push_back(Op{OP_REGAUGE_APPLY, 0, 0, 0, "regauge_apply_in_place"});
  }
  if (hp.refresh_period_T > 1) plan_lowrank_project_fast(c);
}

template <class T>
size_t bytes_of(const std::vector<T>& v) { return align_up(v.size() * sizeof(T)); }

// ---------------------------------------------------------------------------
// The library's own scratch buffer, for callers that cannot allocate device memory (adapm_step_static).  Every GPU
// the library runs on holds one copy of the array at its own address until the process ends.  In host code the
// array's NAME is only a stand-in for the symbol, not a device address: host code uses the pointer that
// hipGetSymbolAddress returned for the device in question, looked up once per device at set-up.
// ---------------------------------------------------------------------------
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)64 << 20;
constexpr int MAX_DEVICES = 64;
char* g_scratch_ptr[MAX_DEVICES] = {nullptr};
const adapm_ctx* g_scratch_user[MAX_DEVICES] = {nullptr};     // context whose step used a device's scratch array last
}  // namespace
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
namespace {

// Address of the scratch array on device `dev` (which must be the current device); looked up on first use.
adapm_status_t scratch_address(int dev, char** out) {
  if (dev < 0 || dev >= MAX_DEVICES) return fail(ADAPM_EINVAL, "device index %d out of range", dev);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(ADAPM_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = (char*)p;
  }
  if (out) *out = g_scratch_ptr[dev];
  return ADAPM_OK;
}


adapm_status_t ensure_uploaded(adapm_ctx* c) {
  if (c->uploaded) return ADAPM_OK;
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  const size_t nb = c->table.size();
  size_t total = bytes_of(c->blocks.h) + bytes_of(c->sk.h) + bytes_of(c->lrb.h) + bytes_of(c->qs.h) + bytes_of(c->proj_keep.h) +
                 bytes_of(c->sprob.h) + bytes_of(c->gn.h) + bytes_of(c->grp.h) + bytes_of(c->rg_apply.h) +
                 adapm_ctx::NSLOT * align_up(2 * nb * sizeof(void*));
  for (auto& l : c->cp) total += bytes_of(l.h);
  for (auto& l : c->rub) total += bytes_of(l.h);
  for (auto& l : c->qt) total += bytes_of(l.h);
  for (auto& l : c->ru) total += bytes_of(l.h);
  for (auto& l : c->chol) total += bytes_of(l.h);
  for (auto& l : c->ew) total += bytes_of(l.h);
  for (auto& l : c->img) total += bytes_of(l.h);
  for (auto& l : c->sit) total += bytes_of(l.h);
  for (auto& l : c->gram) total += bytes_of(l.h);
  for (auto& l : c->gfin) total += bytes_of(l.h);
  for (auto& l : c->gnorm) total += bytes_of(l.h);
  for (int i = 0; i < 12; ++i) total += bytes_of(c->proj[i].h);
  for (int i = 0; i < 2; ++i) total += bytes_of(c->vs[i].h) + bytes_of(c->vf[i].h);
  for (auto& g : c->gemms) total += bytes_of(g.probs) + bytes_of(g.tiles);
  HIP_TRY(hipMalloc((void**)&c->arena, total));
  size_t off = 0;
  hipError_t err = hipSuccess;
  auto put = [&](const void* src, size_t n) -> void* {
    void* dst = c->arena + off;
    if (n && err == hipSuccess) err = hipMemcpy(dst, src, n, hipMemcpyHostToDevice);
    off += align_up(n);
    return dst;
  };
#define PUT_LIST(L) (L).d = (decltype((L).d))put((L).h.data(), (L).h.size() * sizeof((L).h[0]))
  PUT_LIST(c->blocks); PUT_LIST(c->sk); PUT_LIST(c->lrb); PUT_LIST(c->qs); PUT_LIST(c->proj_keep); PUT_LIST(c->sprob); PUT_LIST(c->gn); PUT_LIST(c->grp); PUT_LIST(c->rg_apply);
  for (auto& l : c->cp) PUT_LIST(l);
  for (auto& l : c->rub) PUT_LIST(l);
  for (auto& l : c->qt) PUT_LIST(l);
  for (auto& l : c->ru) PUT_LIST(l);
  for (auto& l : c->chol) PUT_LIST(l);
  for (auto& l : c->ew) PUT_LIST(l);
  for (auto& l : c->img) PUT_LIST(l);
  for (auto& l : c->sit) PUT_LIST(l);
  for (auto& l : c->gram) PUT_LIST(l);
  for (auto& l : c->gfin) PUT_LIST(l);
  for (auto& l : c->gnorm) PUT_LIST(l);
  for (int i = 0; i < 12; ++i) PUT_LIST(c->proj[i]);
  for (int i = 0; i < 2; ++i) { PUT_LIST(c->vs[i]); PUT_LIST(c->vf[i]); }
#undef PUT_LIST
  for (auto& g : c->gemms) {
    g.d_probs = (GemmProblem*)put(g.probs.data(), g.probs.size() * sizeof(GemmProblem));
    g.d_tiles = (GemmTile*)put(g.tiles.data(), g.tiles.size() * sizeof(GemmTile));
  }
  if (err != hipSuccess) return fail(ADAPM_EHIP, "plan upload: %s", hipGetErrorString(err));
  void** stage = nullptr;
  HIP_TRY(hipHostMalloc((void**)&stage, adapm_ctx::NSLOT * 2 * nb * sizeof(void*), hipHostMallocDefault));
  for (int k = 0; k < adapm_ctx::NSLOT; ++k) {
    c->slot[k].d = (void**)(c->arena + off);
    off += align_up(2 * nb * sizeof(void*));
    c->slot[k].h = stage + (size_t)k * 2 * nb;
    HIP_TRY(hipEventCreateWithFlags(&c->slot[k].copied, hipEventDisableTiming));
  }
  // set-up also looks up this device's copy of the library's scratch array (adapm_step_static)
  adapm_status_t st = scratch_address(dev, nullptr);
  if (st != ADAPM_OK) return st;
  c->device = dev;
  c->uploaded = true;
  return ADAPM_OK;
}

bool is_refresh(const adapm_ctx* c, int64_t step) {
  return c->hp.refresh_period_T <= 1 || (step - 1) % c->hp.refresh_period_T == 0;
}

// Device-resident pointer table of this call: the slot that already holds these pointers, or the least recently
// used one rewritten by a copy on the step's stream.
adapm_status_t pointer_table(adapm_ctx* c, void* const* params_dev, const void* const* grads_dev, hipStream_t s,
                             void*** out) {
  const size_t nb = c->table.size();
  adapm_ctx::PtrSlot* hit = nullptr;
  adapm_ctx::PtrSlot* lru = nullptr;        // an empty slot if there is one, else the least recently used
  for (adapm_ctx::PtrSlot& q : c->slot) {
    if (q.valid && memcmp(q.h, params_dev, nb * sizeof(void*)) == 0 && memcmp(q.h + nb, grads_dev, nb * sizeof(void*)) == 0) {
      hit = &q;
      break;
    }
    if (!lru || (!q.valid && lru->valid) || (q.valid == lru->valid && q.last_use < lru->last_use)) lru = &q;
  }
  if (!hit) {
    hit = lru;
    if (hit->valid) {
      // the pinned copy was the source of an earlier upload; NSLOT - 1 uploads later that has long finished
      const hipError_t q = hipEventQuery(hit->copied);
      (void)hipGetLastError();
      if (q == hipErrorNotReady) HIP_TRY(hipEventSynchronize(hit->copied));
      else if (q != hipSuccess) return fail(ADAPM_EHIP, "hipEventQuery: %s", hipGetErrorString(q));
    }
    memcpy(hit->h, params_dev, nb * sizeof(void*));
    memcpy(hit->h + nb, grads_dev, nb * sizeof(void*));
    HIP_TRY(hipMemcpyAsync(hit->d, hit->h, 2 * nb * sizeof(void*), hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(hit->copied, s));
    hit->valid = true;
  }
  hit->last_use = ++c->use_clock;
  *out = hit->d;
  return ADAPM_OK;
}

const Op kGradNormOp = {OP_GRADNORM, 0, 0, 0, "grad_norm"};

adapm_status_t run_op(adapm_ctx* c, const Op& op, Bases& bs, const StepScalars& sc, double* partials, void* state_dev,
                      void* workspace_dev, hipStream_t s, int64_t& launches) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool skipped = false;
  if (c->profiling) {
    for (hipEvent_t* e : {&e0, &e1}) {
      if (!c->event_pool.empty()) { *e = c->event_pool.back(); c->event_pool.pop_back(); }
      else HIP_TRY(hipEventCreate(e));
    }
    HIP_TRY(hipEventRecord(e0, s));
  }
  switch (op.kind) {
    case OP_GRADNORM: {
      // sums of squares of every gradient (unscaled), then norm and factor; every later kernel reads the factor
      double* gp = (double*)(bs.ws + c->off_gn_partials);
      float* out = (float*)(bs.ws + c->off_gn_out);
      launch_vstat(c->blocks.d, c->gn.d, (int64_t)c->gn.h.size(), gp, bs, sc.beta2, s);
      launch_gradnorm_final(gp, (int64_t)c->gn.h.size(), c->grad_clip, out, s);
      bs.gscale = out + 1;
      ++launches;
      break;
    }
    case OP_VSTAT:
      launch_vstat(c->blocks.d, c->vs[op.index].d, (int64_t)c->vs[op.index].h.size(), partials, bs, sc.beta2, s);
      break;
    case OP_VFINAL:
      launch_vfinal(c->blocks.d, c->vf[op.index].d, (int64_t)c->vf[op.index].h.size(), partials, bs, sc.beta2, s);
      break;
    case OP_UPDATE: {
      StepScalars x = sc;
      x.cG = op.cG; x.cC = op.cC;
      launch_update(c->blocks.d, c->ew[op.index].d, (int64_t)c->ew[op.index].h.size(), bs, x, s);
      break;
    }
    case OP_GEMM: {
      const GemmList& g = c->gemms[op.index];
      launch_gemm64(g.d_probs, g.d_tiles, (int64_t)g.tiles.size(), bs, s);
      break;
    }
    case OP_GEMM_MFMA: {
      const GemmList& g = c->gemms[op.index];
      launch_gemm_mfma(g.d_probs, g.d_tiles, (int64_t)g.tiles.size(), bs, s);
      break;
    }
    case OP_CHOL:
      launch_chol(c->chol[op.index].d, (int64_t)c->chol[op.index].h.size(), bs, s);
      break;
    case OP_QSPLIT:
      // index 1: only needed if the copies in the workspace are not the ones written last
      if (op.index == 1 && c->split_ws == workspace_dev && c->split_state == state_dev) { skipped = true; break; }
      launch_qimage(c->qs.d, (int64_t)c->qs.h.size(), c->lrb.d, bs, s);
      c->split_ws = workspace_dev;
      c->split_state = state_dev;
      break;
    case OP_QFIMG:
      launch_qf_image(c->img[op.index].d, (int64_t)c->img[op.index].h.size(), bs, s);
      break;
    case OP_STRIPE:
      launch_stripe(1 << ((op.index % 6) >> 1), (op.index & 1) != 0, c->sit[op.index].d, (int64_t)c->sit[op.index].h.size(), c->sprob.d, bs, s);
      break;
    case OP_UPDATE_GROUPED:
      launch_update_grouped(c->blocks.d, c->grp.d, (int64_t)c->grp.h.size(), bs, sc, s);
      break;
    case OP_COPY:
      launch_copy(c->cp[op.index].d, (int64_t)c->cp[op.index].h.size(), bs, s);
      break;
    case OP_GNORM:
      launch_gram_norm(c->gnorm[op.index].d, (int64_t)c->gnorm[op.index].h.size(), bs, s);
      break;
    case OP_REGAUGE_APPLY:
      launch_regauge_apply(c->rg_apply.d, (int64_t)c->rg_apply.h.size(), bs, s);
      break;
    case OP_GRAM_FIN:
      launch_gram_finish(c->gfin[op.index].d, (int64_t)c->gfin[op.index].h.size(), bs, s);
      break;
    case OP_GRAM:
      launch_gram(c->gram[op.index].d, (int64_t)c->gram[op.index].h.size(), bs, s);
      break;
    case OP_QTIMG:
      launch_qt_image(c->qt[op.index].d, (int64_t)c->qt[op.index].h.size(), bs, s);
      break;
    case OP_REFRESH_UPDATE: {
      StepScalars x = sc;
      x.cG = op.cG; x.cC = op.cC;
      launch_refresh_update(1 << ((op.index % 6) >> 1), (op.index & 1) != 0, c->ru[op.index].d, (int64_t)c->ru[op.index].h.size(),
                            c->rub[op.aux].d, bs, x, s);
      break;
    }
    case OP_PROJ_KEEP: {
      StepScalars x = sc;
      x.cG = c->hp.bias_correction ? 1.f : 0.f;
      x.cC = 1.f;
      launch_proj_keep(c->proj_keep.d, (int64_t)c->proj_keep.h.size(), c->lrb.d, bs, x, s);
      break;
    }
    case OP_PROJ: {
      StepScalars x = sc;
      x.cG = c->hp.bias_correction ? 1.f : 0.f;
      x.cC = 1.f;
      launch_proj(1 << ((op.index >> 1) % 3), (op.index & 1) != 0, op.index >= 6, c->proj[op.index].d,
                  (int64_t)c->proj[op.index].h.size(), c->lrb.d, bs, x, s);
      break;
    }
  }
  if (c->profiling) {
    if (skipped) { c->event_pool.push_back(e0); c->event_pool.push_back(e1); }
    else {
      HIP_TRY(hipEventRecord(e1, s));
      c->prof.push_back(ProfRec{op.label, e0, e1});
    }
  }
  if (!skipped) ++launches;
  return ADAPM_OK;
}

// The launches of one step on stream s.  Arguments were validated by the entry point; the plan is on the device.
// Allocates nothing unless per-launch timing is switched on (event records).
adapm_status_t enqueue_step(adapm_ctx* c, void* const* params_dev, const void* const* grads_dev, void* state_dev,
                            void* workspace_dev, int64_t step, float lr, hipStream_t s) {
  const size_t nb = c->table.size();
  void** table = nullptr;
  adapm_status_t st = pointer_table(c, params_dev, grads_dev, s, &table);
  if (st != ADAPM_OK) return st;

  Bases bs;
  bs.state = (char*)state_dev;
  bs.ws = (char*)workspace_dev;
  bs.params = (void* const*)table;
  bs.grads = (const void* const*)(table + nb);
  bs.gscale = nullptr;

  StepScalars sc;
  sc.beta1 = c->hp.beta1; sc.beta2 = c->hp.beta2; sc.eps = c->hp.eps; sc.clip = c->hp.clip;
  sc.lr = lr;
  sc.inv_debias_m = sc.inv_debias_v = 1.f;
  if (c->hp.adam_debias) {
    sc.inv_debias_m = (float)(1.0 / (1.0 - std::pow((double)c->hp.beta1, (double)step)));
    sc.inv_debias_v = (float)(1.0 / (1.0 - std::pow((double)c->hp.beta2, (double)step)));
  }
  sc.cG = sc.cC = 0.f;
  // step with R held: D = beta1 (L' - P) with eq. 4, or D = L_t without it
  sc.dL = c->hp.beta1;
  sc.dP = c->hp.bias_correction ? -c->hp.beta1 : 1.f - c->hp.beta1;

  double* partials = c->off_partials >= 0 ? (double*)(bs.ws + c->off_partials) : nullptr;
  int64_t launches = 0;
  const bool refresh = is_refresh(c, step);
  if (c->grad_clip > 0.f && std::isfinite(c->grad_clip)) {
    st = run_op(c, kGradNormOp, bs, sc, partials, state_dev, workspace_dev, s, launches);
    if (st != ADAPM_OK) return st;
  }
  for (const Op& op : (refresh ? c->seq_refresh : c->seq_project)) {
    st = run_op(c, op, bs, sc, partials, state_dev, workspace_dev, s, launches);
    if (st != ADAPM_OK) return st;
  }
  if (refresh && c->hp.refresh_period_T > 1) c->gauge_ok = true;
  c->last_launches = launches;
  HIP_TRY(hipGetLastError());
  return ADAPM_OK;
}

}  // namespace

// ===========================================================================
// C ABI
// ===========================================================================
extern "C" {

const char* adapm_last_error(void) { return g_err.c_str(); }

adapm_status_t adapm_init(adapm_ctx** out, const adapm_block_t* table, int64_t nblocks, const adapm_hparams_t* hp) {
  if (!out) return fail(ADAPM_EINVAL, "out is null");
  *out = nullptr;
  adapm_status_t st = validate(table, nblocks, hp);
  if (st != ADAPM_OK) return st;
  adapm_ctx* c = new (std::nothrow) adapm_ctx();
  if (!c) return fail(ADAPM_ENOMEM, "out of host memory");
  try {
    c->table.assign(table, table + nblocks);
    c->hp = *hp;
    const char* nk = getenv("ADAPM_PROJ_KEEP");
    c->keep_enabled = nk && nk[0] == '1';
    build_plan(c);
  } catch (const std::bad_alloc&) {
    delete c;
    return fail(ADAPM_ENOMEM, "out of host memory while planning");
  }
  *out = c;
  return ADAPM_OK;
}

size_t adapm_state_bytes(const adapm_ctx* c) { return c ? c->state_bytes : 0; }
size_t adapm_workspace_bytes(const adapm_ctx* c) { return c ? c->ws_bytes : 0; }

adapm_status_t adapm_state_offsets(const adapm_ctx* c, int64_t block, size_t* L, size_t* R, size_t* m, size_t* v) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (block < 0 || block >= (int64_t)c->table.size()) return fail(ADAPM_EINVAL, "block index out of range");
  const Layout& l = c->lay[block];
  if (L) *L = (size_t)l.sL;
  if (R) *R = (size_t)l.sR;
  if (m) *m = (size_t)l.sm;
  if (v) *v = (size_t)l.sv;
  return ADAPM_OK;
}

adapm_status_t adapm_state_init(adapm_ctx* c, void* state_dev, void* stream) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (!state_dev && c->state_bytes) return fail(ADAPM_EINVAL, "state_dev is null");
  if ((uintptr_t)state_dev & 15) return fail(ADAPM_EINVAL, "state_dev must be 16-byte aligned");
  adapm_status_t st = ensure_uploaded(c);
  if (st != ADAPM_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  c->split_ws = nullptr;
  c->gauge_ok = false;
  launch_fill_zero(state_dev, c->state_bytes, s);
  launch_sketch(c->sk.d, (int64_t)c->sk.h.size(), (char*)state_dev, s);
  HIP_TRY(hipGetLastError());
  return ADAPM_OK;
}

adapm_status_t adapm_step(adapm_ctx* c, void* const* params_dev, const void* const* grads_dev, void* state_dev,
                          void* workspace_dev, int64_t step, float lr, void* stream) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (step < 1) return fail(ADAPM_ESTATE, "step must be >= 1 (got %lld)", (long long)step);
  if (!params_dev || !grads_dev) return fail(ADAPM_EINVAL, "params_dev / grads_dev is null");
  if (!state_dev || ((uintptr_t)state_dev & 15)) return fail(ADAPM_EINVAL, "state_dev is null or misaligned");
  if (c->ws_bytes && (!workspace_dev || ((uintptr_t)workspace_dev & 255)))
    return fail(ADAPM_EINVAL, "workspace_dev is null or not 256-byte aligned");
  const size_t nb = c->table.size();
  for (size_t i = 0; i < nb; ++i) {
    if (!params_dev[i] || !grads_dev[i]) return fail(ADAPM_EINVAL, "block %zu: null parameter or gradient pointer", i);
    if (((uintptr_t)params_dev[i] | (uintptr_t)grads_dev[i]) & 15)
      return fail(ADAPM_EINVAL, "block %zu: parameter / gradient pointer not 16-byte aligned", i);
  }
  const bool refresh = is_refresh(c, step);
  if (!refresh && c->n_lowrank > 0 && !c->gauge_ok)
    return fail(ADAPM_ESTATE, "step %lld holds R, but this state's R has not been orthonormalised yet: run a step with "
                "(step - 1) %% refresh_period_T == 0 first, or call adapm_state_loaded() after restoring a checkpoint",
                (long long)step);
  adapm_status_t st = ensure_uploaded(c);     // a no-op after adapm_state_init
  if (st != ADAPM_OK) return st;
  return enqueue_step(c, params_dev, grads_dev, state_dev, workspace_dev, step, lr, (hipStream_t)stream);
}

adapm_status_t adapm_step_static(adapm_ctx* c, void* const* params_dev, const void* const* grads_dev, void* state_dev,
                                 int64_t step, float lr, void* stream) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (step < 1) return fail(ADAPM_ESTATE, "step must be >= 1 (got %lld)", (long long)step);
  if (!params_dev || !grads_dev) return fail(ADAPM_EINVAL, "params_dev / grads_dev is null");
  if (!state_dev || ((uintptr_t)state_dev & 15)) return fail(ADAPM_EINVAL, "state_dev is null or misaligned");
  if (c->ws_bytes > STATIC_SCRATCH_BYTES)
    return fail(ADAPM_EINVAL, "this table needs %zu bytes of scratch, the library's own buffer holds %zu: use adapm_step "
                "with a caller-allocated workspace", c->ws_bytes, STATIC_SCRATCH_BYTES);
  const size_t nb = c->table.size();
  for (size_t i = 0; i < nb; ++i) {
    if (!params_dev[i] || !grads_dev[i]) return fail(ADAPM_EINVAL, "block %zu: null parameter or gradient pointer", i);
    if (((uintptr_t)params_dev[i] | (uintptr_t)grads_dev[i]) & 15)
      return fail(ADAPM_EINVAL, "block %zu: parameter / gradient pointer not 16-byte aligned", i);
  }
  if (!c->uploaded)
    return fail(ADAPM_ESTATE, "adapm_step_static allocates nothing: run adapm_state_init on this context first (it places "
                "the launch plan on the device)");
  if (c->profiling) return fail(ADAPM_ESTATE, "per-launch timing creates events: switch it off for adapm_step_static");
  const bool refresh = is_refresh(c, step);
  if (!refresh && c->n_lowrank > 0 && !c->gauge_ok)
    return fail(ADAPM_ESTATE, "step %lld holds R, but this state's R has not been orthonormalised yet", (long long)step);
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != c->device) return fail(ADAPM_ESTATE, "the context was set up on device %d, the current device is %d", c->device, dev);
  char* ws = nullptr;
  adapm_status_t st = scratch_address(dev, &ws);      // a table look-up: the address was resolved at set-up
  if (st != ADAPM_OK) return st;
  // the array is shared by every context on this device: whatever another context (or another state buffer of this
  // one, see the workspace rule of adapm_step) left there is not ours
  if (g_scratch_user[dev] != c) c->split_ws = nullptr;
  g_scratch_user[dev] = c;
  return enqueue_step(c, params_dev, grads_dev, state_dev, ws, step, lr, (hipStream_t)stream);
}

size_t adapm_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

adapm_status_t adapm_profile_enable(adapm_ctx* c, int32_t on) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  c->profiling = on != 0;
  return ADAPM_OK;
}

int64_t adapm_profile_read(adapm_ctx* c, int64_t index, char* name, size_t name_cap, double* total_ms,
                           int64_t* launches) {
  if (!c) return 0;
  // fold the finished event pairs into per-label totals (the caller has synchronised the stream)
  auto& agg = c->prof_agg;
  if (index == 0) {
    agg.clear();
    for (const ProfRec& r : c->prof) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) ms = 0.f;
      c->event_pool.push_back(r.e0);
      c->event_pool.push_back(r.e1);
      bool found = false;
      for (auto& a : agg)
        if (a.first == r.label) { a.second.first += ms; a.second.second += 1; found = true; break; }
      if (!found) agg.push_back({r.label, {ms, 1}});
    }
    c->prof.clear();
  }
  if (index < 0 || index >= (int64_t)agg.size()) return (int64_t)agg.size();
  if (name && name_cap) { strncpy(name, agg[index].first.c_str(), name_cap - 1); name[name_cap - 1] = 0; }
  if (total_ms) *total_ms = agg[index].second.first;
  if (launches) *launches = agg[index].second.second;
  return (int64_t)agg.size();
}

adapm_status_t adapm_state_loaded(adapm_ctx* c) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  c->split_ws = nullptr;
  c->gauge_ok = true;      // the caller vouches for the restored state: a checkpoint taken with T > 1 holds an orthonormal R
  return ADAPM_OK;
}

adapm_status_t adapm_set_grad_clip(adapm_ctx* c, float max_norm) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (std::isnan(max_norm)) return fail(ADAPM_EINVAL, "max_norm is NaN");
  c->grad_clip = (max_norm > 0.f && std::isfinite(max_norm)) ? max_norm : 0.f;
  return ADAPM_OK;
}

adapm_status_t adapm_last_grad_norm(adapm_ctx* c, const void* workspace_dev, void* stream, float* norm, float* scale) {
  if (!c) return fail(ADAPM_EINVAL, "ctx is null");
  if (c->off_gn_out < 0) return fail(ADAPM_ESTATE, "no plan");
  if (!workspace_dev) {      // the step ran on the library's own scratch array
    char* ws = nullptr;
    if (!c->uploaded || scratch_address(c->device, &ws) != ADAPM_OK) return fail(ADAPM_ESTATE, "no step has run on this context");
    workspace_dev = ws;
  }
  float h[2] = {0.f, 1.f};
  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(hipMemcpyAsync(h, (const char*)workspace_dev + c->off_gn_out, sizeof h, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (norm) *norm = h[0];
  if (scale) *scale = h[1];
  return ADAPM_OK;
}

float adapm_lr_cosine_warmup(int64_t step, float peak_lr, float min_lr, int64_t warmup_steps, int64_t total_steps) {
  if (warmup_steps > 0 && step <= warmup_steps) return (float)((double)peak_lr * (double)step / (double)warmup_steps);
  if (step >= total_steps) return min_lr;
  const double x = (double)(step - warmup_steps) / (double)(total_steps - warmup_steps);
  return (float)((double)min_lr + 0.5 * ((double)peak_lr - (double)min_lr) * (1.0 + std::cos(M_PI * x)));
}

int32_t adapm_block_contraction(const adapm_ctx* c, int64_t block) {
  if (!c || block < 0 || block >= (int64_t)c->lay.size()) return -1;
  const int path = c->lay[block].path;
  return path == PATH_FAST ? ADAPM_CONTRACT_BF16X2 : (path == PATH_F64 ? ADAPM_CONTRACT_F64 : -1);
}

int64_t adapm_last_launch_count(const adapm_ctx* c) { return c ? c->last_launches : 0; }

double adapm_algorithmic_bytes(const adapm_ctx* c, int32_t refresh_step) {
  if (!c) return 0.0;
  const bool refresh = refresh_step != 0 || c->hp.refresh_period_T <= 1;
  double tot = 0.0;
  for (const adapm_block_t& b : c->table) {
    const double mn = (double)b.rows * (double)b.cols;
    tot += mn * (esize(b.grad_dtype) + 2.0 * esize(b.param_dtype));
    if (b.mom_mode == ADAPM_MOM_FULL) tot += 8.0 * mn;
    if (b.mom_mode == ADAPM_MOM_LOWRANK) {
      const double m = (double)b.rows, n = (double)b.cols, r = b.rank;
      tot += refresh ? 8.0 * (m + n) * r : 8.0 * m * r + 4.0 * r * n;
    }
    tot += 8.0 * (double)num_v(b);
  }
  return tot;
}

double adapm_algorithmic_flops(const adapm_ctx* c, int32_t refresh_step) {
  if (!c) return 0.0;
  const bool refresh = refresh_step != 0 || c->hp.refresh_period_T <= 1;
  const double n_eff = (double)effective_step_sizes(c->hp.refresh_iters_K).size();
  double tot = 0.0;
  for (const adapm_block_t& b : c->table) {
    if (b.mom_mode != ADAPM_MOM_LOWRANK) continue;
    const double m = (double)b.rows, n = (double)b.cols, r = b.rank;
    if (refresh) tot += n_eff * (4.0 * m * n * r + 8.0 * r * r * (m + n)) + (c->hp.bias_correction ? 4.0 : 2.0) * m * n * r;
    else tot += 4.0 * m * n * r;
  }
  return tot;
}

void adapm_destroy(adapm_ctx* c) {
  if (!c) return;
  for (const adapm_ctx*& u : g_scratch_user)
    if (u == c) u = nullptr;
  if (c->uploaded) {
    for (adapm_ctx::PtrSlot& q : c->slot)
      if (q.copied) { (void)hipEventSynchronize(q.copied); (void)hipEventDestroy(q.copied); }
    if (c->slot[0].h) (void)hipHostFree(c->slot[0].h);      // one pinned allocation shared by the slots
    for (const ProfRec& r : c->prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
    if (c->arena) (void)hipFree(c->arena);
  }
  delete c;
}

}  // extern "C"
